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
        if enc == BIPOLAR:
            x[1, :4] = [0.0, -0.0, 0.2 * scale[0], -0.2 * scale[0]]  # no zero level: the sign decides, zero is +1
        q = oracle.quantize(x, scale, bits, enc)
        got = dlrt.dlrt_pack_bitplanes(dev(x), bits, enc, scale=dev(scale))
        assert np.array_equal(words(got), oracle.pack_bitplanes(q, bits, enc))


@pytest.mark.parametrize("Co,k,Ci", [(3, 3, 40), (16, 1, 32), (5, 5, 7), (7, 3, 100), (8, 1, 256)])
def test_pack_conv_weights_float_source_quantizes_like_the_oracle(dlrt, oracle, Co, k, Ci):
    """Section IV's quantizer in front of the conv-weight packer: ragged channel counts (a tap's last word is
    partly padding), ties, saturation at both ends, every encoding, one scale for the tensor."""
    r = rng(4100 + Co * 7 + Ci)
    for bits, enc in [(2, TWOS), (1, BIPOLAR), (4, TWOS), (3, UNSIGNED), (1, TWOS)]:
        s = np.float32(r.uniform(0.05, 0.9))
        x = r.normal(0, 2.0 * s, size=(Co, k, k, Ci)).astype(np.float32)
        flat = x.reshape(-1)
        flat[:10] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 1e9, -1e9, 0.0, -0.0], np.float32) * s
        flat[-1] = np.float32(-1e9)  # the last element of the last tap saturates too
        q = oracle.quantize(x.reshape(Co * k * k, Ci), np.array([s], np.float32), bits, enc).reshape(x.shape)
        got = dlrt.dlrt_pack_conv_weights(dev(x), bits, enc, scale=dev(np.array([s], np.float32)))
        assert got.shape == (Co, bits, k * k * ((Ci + 31) // 32))
        assert np.array_equal(words(got), oracle.pack_conv_weights(q, bits, enc)), (bits, enc)


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
def test_gemm_config5_full_size_every_output(dlrt, oracle, abits, wbits, enc_w):
    """4096^3 in the configuration the benchmark times, all 16.8 M outputs against the oracle (a few
    seconds of host time per pair), plus the row-sum / column-sum identities, which hold at any size:
    sum_n C[m,n] = a[m,:] . (sum_n w[n,:]) and sum_m C[m,n] = (sum_m a[m,:]) . w[n,:]."""
    c, a, w = inputs.config5(abits, wbits)
    if enc_w == BIPOLAR:
        w = inputs.uniform_values(w.shape, 1, BIPOLAR, inputs.seed_for(5, 1) + 7)
    got = gpu_gemm(dlrt, a, w, abits, wbits, c.enc_a, enc_w)
    assert np.array_equal(got, oracle.gemm_i32(a, w))
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


ACT_SCALE = 0.8  # step size of the quantizer that reads a float32 layer


def oracle_stack(oracle, config, layers, wbits, enc_w, abits=2, batch=1, f32_layers=()):
    """Oracle pass, layer by layer, producing the frozen scale / bias arrays both sides use.  abits,
    wbits and enc_w are one value or one per layer; a layer's output takes the width its readers expect."""
    n = len(layers)
    ab = list(abits) if isinstance(abits, (list, tuple)) else [abits] * n
    wb = list(wbits) if isinstance(wbits, (list, tuple)) else [wbits] * n
    ew = list(enc_w) if isinstance(enc_w, (list, tuple)) else [enc_w] * n
    qb = [next((ab[j] for j in range(n) if layers[j].src == i), ab[i]) for i in range(n)]
    L0 = layers[0]
    x0 = inputs.uniform_values((batch, L0.H, L0.W, L0.Ci), ab[0], UNSIGNED, inputs.seed_for(config, 0))
    weights = [inputs.uniform_values((L.Co, L.k, L.k, L.Ci), wb[i], ew[i], inputs.seed_for(config, 1, layer=i))
               for i, L in enumerate(layers)]
    ref_acc, ref_q, scales, biases, ref_y = [], [], [], [], {}
    for i, L in enumerate(layers):
        xin = x0 if L.src < 0 else ref_q[L.src]
        acc = oracle.conv2d_i32(xin.astype(np.int8), weights[i], (L.stride, L.stride), (L.pad, L.pad))
        s, b = calibrate(acc)
        levels = 1 << qb[i]
        s, b = (s * levels / 4).astype(np.float32), (b * levels / 4).astype(np.float32)
        if i in f32_layers:  # the layer stays float32; its readers quantize it (Section IV)
            ref_y[i], _ = oracle.epilogue_f32(acc, s, b)
            q = oracle.quantize(ref_y[i].reshape(-1, L.Co), np.float32(ACT_SCALE), qb[i], UNSIGNED)
            q = q.reshape(acc.shape).astype(np.uint8)
        else:
            _, q = oracle.epilogue_f32(acc, s, b, qbits=qb[i])
        hist = np.bincount(q.ravel(), minlength=levels) / q.size
        # the chain must not degenerate to a constant: the values stay spread over the levels
        assert hist.max() < 0.75 and (hist >= 0.02).sum() >= min(levels, 4), (L.name, hist)
        ref_acc.append(acc), ref_q.append(q), scales.append(s), biases.append(b)
    return x0, weights, ref_acc, ref_q, scales, biases, qb, ref_y


def run_stack_against_oracle(dlrt, oracle, config, layers, wbits, enc_w, fused, graph=False, abits=2, batch=1,
                             f32_layers=()):
    from paper_2207_08820_amd.stack import ConvStack

    x0, weights, ref_acc, ref_q, scales, biases, qb, ref_y = oracle_stack(oracle, config, layers, wbits, enc_w, abits,
                                                                          batch, f32_layers)
    stack = ConvStack(layers, weights, scales, biases, abits, wbits, enc_w, device=DEV, fused=fused, batch=batch,
                      f32_layers=f32_layers, act_scales={i: ACT_SCALE for i in f32_layers})
    assert stack.qbits == qb
    x0_dev = dev(x0.astype(np.uint8))
    if graph:
        stack.capture(x0_dev)
    replays = 3 if graph else 1
    for rep in range(replays):
        if graph:
            for pl in stack.layers:  # eager work between replays: wipe what the graph must rewrite
                pl.acc.zero_(), pl.q.zero_(), pl.out_packed.zero_()
            torch.cuda.synchronize()
            stack.replay()
        else:
            stack.run(x0_dev)
        torch.cuda.synchronize()
        for i, L in enumerate(layers):
            assert np.array_equal(stack.layers[i].acc.cpu().numpy(), ref_acc[i]), (L.name, rep)
            if i in f32_layers:
                assert np.array_equal(stack.layers[i].y.cpu().numpy(), ref_y[i]), (L.name, rep)
            else:
                assert np.array_equal(stack.layers[i].q.cpu().numpy(), ref_q[i]), (L.name, rep)
            if fused or i in f32_layers:
                want = oracle.pack_bitplanes(ref_q[i].reshape(-1, L.Co).astype(np.int8), qb[i], UNSIGNED)
                assert np.array_equal(words(stack.layers[i].out_packed), want), (L.name, rep)


@pytest.mark.parametrize("fused", [False, True])
def test_config3_resnet18_stack_every_layer_bit_exact(dlrt, oracle, fused):
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS, fused)


@pytest.mark.parametrize("fused", [False, True])
def test_config4_yolo_style_stack_bipolar_weights_every_layer_bit_exact(dlrt, oracle, fused):
    run_stack_against_oracle(dlrt, oracle, 4, inputs.yolo_style_stack(), 1, BIPOLAR, fused)


@pytest.mark.parametrize("fused", [False, True])
def test_resnet18_stack_1a2w_as_in_the_papers_vww_experiment(dlrt, oracle, fused):
    """1-bit activations with 2-bit weights, the paper's second ResNet18 precision (Section VII-A)."""
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS, fused, abits=1)


@pytest.mark.parametrize("fused", [False, True])
def test_resnet18_stack_mixed_precision_per_layer(dlrt, oracle, fused):
    """Per-layer precision lists (the paper keeps sensitive layers at higher precision, Section VII-D):
    stage 0 at A4W4, stage 1 at A3W2 unsigned weights, stage 2 at A2W2, stage 3 at A2 with bipolar W1."""
    layers = inputs.resnet18_stack()
    ab, wb, ew = [], [], []
    for L in layers:
        stage = int(L.name[1])
        a, w, e = [(4, 4, TWOS), (3, 2, UNSIGNED), (2, 2, TWOS), (2, 1, BIPOLAR)][stage]
        # a stage's first convs read the previous stage's output: they take that stage's activation width
        if stage > 0 and (L.name.endswith("b0c0_3x3") or "down" in L.name):
            a = [4, 3, 2][stage - 1]
        ab.append(a), wb.append(w), ew.append(e)
    run_stack_against_oracle(dlrt, oracle, 3, layers, wb, ew, fused, abits=ab)


@pytest.mark.parametrize("fused,batch", [(False, 3), (True, 3), (True, 20)])
def test_resnet18_stack_batched(dlrt, oracle, fused, batch):
    """Several images per pass: batch 3 stays on the per-wave kernel (with paired launches), batch 20
    moves the first stages to the block kernel and splits their pairs into two launches."""
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS, fused, batch=batch)


@pytest.mark.parametrize("fused", [False, True])
def test_resnet18_stack_with_float32_pass_through_layers(dlrt, oracle, fused):
    """Layers kept in float32 (the paper leaves precision-sensitive layers unquantized, Section VII-D):
    the first conv, a stride-2 conv with a paired 1x1 beside it, and the last conv emit the dequantized
    float32 result; the quantizer of Section IV, fused into the packer, feeds their readers."""
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS, fused, f32_layers=(0, 4, 18))


@pytest.mark.parametrize("batch", [1, 2])
def test_yolo_style_stack_with_3x3_stride1_bottleneck_convs(dlrt, oracle, batch):
    layers = inputs.yolo_style_stack(bottlenecks=True)
    assert len(layers) == 20
    run_stack_against_oracle(dlrt, oracle, 4, layers, 1, BIPOLAR, True, batch=batch)


def test_yolo_style_stack_batched(dlrt, oracle):
    run_stack_against_oracle(dlrt, oracle, 4, inputs.yolo_style_stack(), 1, BIPOLAR, True, batch=2)


def test_config3_stack_as_hip_graph_every_replay_bit_exact(dlrt, oracle):
    run_stack_against_oracle(dlrt, oracle, 3, inputs.resnet18_stack(), 2, TWOS, fused=True, graph=True)


def test_config4_stack_batched_as_hip_graph_every_replay_bit_exact(dlrt, oracle):
    """The YOLO-style chain at batch 2 in one captured graph: row, block and per-wave kernels and the paired
    launches all sit in the same graph; three replays with eager work between them, each checked."""
    layers = inputs.yolo_style_stack()
    kinds = {dlrt.dlrt_query_plan(2 * L.M, L.Co, L.k * L.k * ((L.Ci + 31) // 32) * 32, 2, 1)["kernel"] for L in layers}
    assert kinds == {"rows", "block", "wave"}
    run_stack_against_oracle(dlrt, oracle, 4, layers, 1, BIPOLAR, fused=True, graph=True, batch=2)


# ---- fused convolution: conv + scale/bias + requant + bitplanes of the result in one launch -------------
def fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=0, ksplit=0, seed=0,
               packed_only=False):
    N, H, W_, Ci = x.shape
    Co, KH, KW, _ = w.shape
    ref = oracle.conv2d_i32(x, w, (stride, stride), (pad, pad))
    scale, bias = calibrate(ref)
    scale = (scale * (1 << qbits) / 4).astype(np.float32)  # spread over the 2^qbits levels
    bias = (bias * (1 << qbits) / 4).astype(np.float32)
    y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=qbits)
    X = dlrt.dlrt_pack_bitplanes(src_tensor(x, ea), abits, ea)
    Wp = dlrt.dlrt_pack_conv_weights(src_tensor(w, ew), wbits, ew)
    Mo = ref.shape[0] * ref.shape[1] * ref.shape[2]
    acc = torch.full(ref.shape, -7, dtype=torch.int32, device=DEV)
    y = torch.full(ref.shape, -7.0, dtype=torch.float32, device=DEV)
    q = torch.full(ref.shape, 99, dtype=torch.uint8, device=DEV)
    packed = torch.full((Mo, qbits, (Co + 31) // 32), -1, dtype=torch.int32, device=DEV)
    tag = (abits, wbits, ea, ew, qbits, tile_rows, ksplit)
    if packed_only:  # the chained-layer call: nothing but the next layer's packed activations
        dlrt.dlrt_bitserial_conv2d_fused(X, Wp, dev(scale), dev(bias), N, H, W_, Ci, Co, KH, KW, (stride, stride),
                                         (pad, pad), abits, wbits, ea, ew, qbits=qbits, out_packed=packed,
                                         tile_rows=tile_rows, ksplit=ksplit)
        torch.cuda.synchronize()
        want = oracle.pack_bitplanes(q_ref.reshape(Mo, Co).astype(np.int8), qbits, UNSIGNED)
        assert np.array_equal(words(packed), want), tag
        return
    dlrt.dlrt_bitserial_conv2d_fused(X, Wp, dev(scale), dev(bias), N, H, W_, Ci, Co, KH, KW, (stride, stride),
                                     (pad, pad), abits, wbits, ea, ew, qbits=qbits, out_acc=acc, out_f32=y, out_q=q,
                                     out_packed=packed, tile_rows=tile_rows, ksplit=ksplit)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref), tag
    assert np.array_equal(y.cpu().numpy(), y_ref), tag
    assert np.array_equal(q.cpu().numpy(), q_ref), tag
    assert np.array_equal(words(packed), oracle.pack_bitplanes(q_ref.reshape(Mo, Co).astype(np.int8), qbits, UNSIGNED)), tag


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_fused_edge_shapes_all_encodings(dlrt, oracle, shape):
    N, H, W, Ci, Co, k, stride, pad = shape
    cases = [(2, 2, UNSIGNED, TWOS, 2), (2, 1, UNSIGNED, BIPOLAR, 2), (1, 1, UNSIGNED, TWOS, 1),
             (4, 4, UNSIGNED, TWOS, 4), (3, 2, TWOS, UNSIGNED, 3), (2, 4, UNSIGNED, TWOS, 2), (3, 3, TWOS, TWOS, 2)]
    for idx, (abits, wbits, ea, ew, qbits) in enumerate(cases):
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 18000 + idx + H)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 19000 + idx + Ci)
        fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits)


ROW_KERNEL_SHAPES = [
    # N, H, W, Ci, Co, k, stride, pad: convs whose im2col row fits a lane's registers (<= 16 words, or 18)
    (1, 9, 7, 32, 32, 1, 1, 0),      # one word, one output word
    (2, 10, 10, 33, 20, 1, 2, 0),    # ragged channels (2 words, the second nearly empty), stride 2, batch 2
    (1, 12, 12, 64, 70, 1, 1, 0),    # ragged output columns: three column words, the last partly filled
    (1, 8, 6, 128, 64, 1, 2, 0),     # four words
    (1, 6, 6, 96, 33, 1, 1, 0),      # three words in a four-word register row
    (1, 5, 5, 160, 129, 1, 1, 0),    # five words in an eight-word register row, 129 columns
    (3, 7, 5, 256, 40, 1, 1, 0),     # eight words, batch 3
    (1, 20, 20, 8, 3, 1, 1, 0),      # a quarter word of channels, three columns, rows beyond one wave
    (1, 11, 9, 32, 40, 3, 1, 1),     # 3x3 over one word of channels: nine words, zero padding at the border
    (2, 10, 10, 20, 33, 3, 2, 1),    # 3x3 stride 2, ragged channels, batch 2
    (1, 9, 9, 3, 16, 3, 1, 0),       # three channels (a stem-like conv), no padding
    (1, 8, 8, 40, 24, 2, 2, 0),      # 2x2 taps of two words: eight words
    (1, 7, 6, 8, 10, 4, 1, 2),       # 4x4 taps: sixteen words, padding wider than one pixel
    (1, 6, 6, 500, 12, 1, 1, 1),     # sixteen words of channels, 1x1 with padding (border outputs are the bias)
    (2, 9, 10, 64, 40, 3, 1, 1),     # 3x3 over two words of channels: eighteen words, batch 2
    (1, 11, 8, 48, 70, 3, 2, 1),     # the same with ragged channels, stride 2 and a ragged third output word
    (2, 9, 10, 64, 96, 3, 1, 1),     # eighteen words, three whole output words (waves of 8 and 16 columns apply)
    (1, 20, 20, 32, 64, 3, 2, 1),    # nine words, two whole output words, stride 2
]


@pytest.mark.parametrize("shape", ROW_KERNEL_SHAPES)
def test_conv_fused_row_kernel_all_encodings(dlrt, oracle, shape):
    """tile_rows = 64 selects the kernel with one output row per lane; ksplit then is the number of
    8-column groups a wave covers (0: planned).  Every output kind, and the packed-only fast path; waves of 8 and
    16 columns (bytes and halves of the output words) exist on that path only, for whole output words and
    unsigned activations, and are refused elsewhere."""
    N, H, W, Ci, Co, k, stride, pad = shape
    cases = [(2, 2, UNSIGNED, TWOS, 2), (2, 1, UNSIGNED, BIPOLAR, 2), (1, 1, UNSIGNED, TWOS, 1),
             (4, 4, UNSIGNED, TWOS, 4), (3, 2, TWOS, UNSIGNED, 3), (2, 4, UNSIGNED, TWOS, 2), (3, 3, TWOS, TWOS, 2)]
    for idx, (abits, wbits, ea, ew, qbits) in enumerate(cases):
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 28000 + idx + H)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 29000 + idx + Ci)
        for groups in (0, 4, 12):
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups)
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups,
                       packed_only=True)
        for groups in (1, 2):
            if Co % 32 == 0 and ea == UNSIGNED:
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups,
                           packed_only=True)
            else:
                with pytest.raises(dlrt.DlrtError):
                    fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64,
                               ksplit=groups, packed_only=True)
            with pytest.raises(dlrt.DlrtError):  # any further output: whole words only
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups)
        with pytest.raises(dlrt.DlrtError):
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=3,
                       packed_only=True)      # 24 columns: neither a part of a word nor whole words


def test_conv_fused_row_kernel_half_width_waves(dlrt, oracle):
    """A negative column-group hint sends out as many units as every die has as two waves of half the width each (the
    planner does this to the last units of a launch of many rounds of waves), the rest as one wave: 50 row blocks
    here, so that every die has units of both kinds.  Halves of whole words with any output, narrower ones
    on the packed-only path."""
    cases = [(2, 2, UNSIGNED, TWOS, 2), (2, 1, UNSIGNED, BIPOLAR, 2), (3, 2, TWOS, UNSIGNED, 3)]
    for idx, (abits, wbits, ea, ew, qbits) in enumerate(cases + cases[:2]):
        # 3200 rows x 64 columns, then a ragged 1517 rows (the last row block a partial one) x 96 columns
        N, H, W, Ci, Co, k, stride, pad = (2, 40, 40, 32, 64, 3, 1, 1) if idx < 3 else (1, 37, 41, 40, 96, 3, 1, 1)
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 28500 + idx)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 29500 + idx)
        fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=-8)
        fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=-8, packed_only=True)
        for groups in (-2, -4):
            if ea == UNSIGNED:
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups,
                           packed_only=True)
            else:
                with pytest.raises(dlrt.DlrtError):
                    fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64,
                               ksplit=groups, packed_only=True)
            with pytest.raises(dlrt.DlrtError):  # any further output: whole words only
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups)
        for groups in (-1, -6):  # halves of 4 or 24 columns: no such wave
            with pytest.raises(dlrt.DlrtError):
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=64, ksplit=groups,
                           packed_only=True)


# (batch, H, W, Ci, Co, k, stride, pad, wbits, weight encoding): layers of the two batched chains that bench.py times,
# one for every kernel and launch form the planner gives them (row kernel with a half-width tail, 32-column row
# kernel on a strided 1x1 conv, panel kernel with one, two and four waves per tile, block kernel)
BATCHED_CHAIN_LAYERS = [
    (64, 56, 56, 64, 64, 3, 1, 1, 2, TWOS),       # 200704 x 64 x 576
    (64, 56, 56, 64, 128, 3, 2, 1, 2, TWOS),      # 50176 x 128 x 576
    (64, 28, 28, 128, 128, 3, 1, 1, 2, TWOS),     # 50176 x 128 x 1152
    (64, 14, 14, 256, 256, 3, 1, 1, 2, TWOS),     # 12544 x 256 x 2304
    (64, 7, 7, 512, 512, 3, 1, 1, 2, TWOS),       # 3136 x 512 x 4608
    (64, 14, 14, 256, 512, 1, 2, 0, 2, TWOS),     # 3136 x 512 x 256
    (16, 160, 160, 64, 128, 3, 2, 1, 1, BIPOLAR), # 102400 x 128 x 576
    (16, 80, 80, 128, 256, 3, 2, 1, 1, BIPOLAR),  # 25600 x 256 x 1152
]


@pytest.mark.parametrize("layer", BATCHED_CHAIN_LAYERS)
def test_batched_chain_layers_at_bench_size_on_sampled_images(dlrt, oracle, layer):
    """The layers of the batched chains at the batch bench.py times them at, launched as the chain launches them
    (planned, nothing but the packed output), against the oracle on whole images of the batch: the first, and
    the eight whose rows fall at the end of a die's share of the launch, where the planner's half-width waves are."""
    B, H, W, Ci, Co, k, stride, pad, wbits, ew = layer
    x = inputs.uniform_values((B, H, W, Ci), 2, UNSIGNED, 31000 + Co + H)
    w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 32000 + Co + H)
    ref0 = oracle.conv2d_i32(x[:1], w, (stride, stride), (pad, pad))
    scale, bias = calibrate(ref0)
    Ho, Wo = ref0.shape[1], ref0.shape[2]
    X = dlrt.dlrt_pack_bitplanes(src_tensor(x, UNSIGNED), 2, UNSIGNED)
    Wp = dlrt.dlrt_pack_conv_weights(src_tensor(w, ew), wbits, ew)
    packed = torch.full((B * Ho * Wo, 2, (Co + 31) // 32), -1, dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_conv2d_fused(X, Wp, dev(scale), dev(bias), B, H, W, Ci, Co, k, k, (stride, stride), (pad, pad),
                                     2, wbits, UNSIGNED, ew, qbits=2, out_packed=packed)
    torch.cuda.synchronize()
    got = words(packed).reshape(B, Ho * Wo, 2, -1)
    for img in [0] + list(range(B // 8 - 1, B, B // 8)):
        ref = oracle.conv2d_i32(x[img:img + 1], w, (stride, stride), (pad, pad))
        _, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=2)
        want = oracle.pack_bitplanes(q_ref.reshape(Ho * Wo, Co).astype(np.int8), 2, UNSIGNED)
        assert np.array_equal(got[img], want.reshape(Ho * Wo, 2, -1)), (layer, img)


PANEL_KERNEL_SHAPES = [
    # N, H, W, Ci, Co, k, stride, pad: convs the panel kernel holds (channels a multiple of 128, so that a tap is
    # whole 16-byte groups), over one, several and ragged numbers of panels, rows beyond one wave, ragged columns
    (1, 9, 7, 128, 32, 3, 1, 1),     # 36 words: three panels of 12
    (2, 10, 10, 128, 20, 3, 2, 1),   # stride 2, batch 2, 20 columns: two full bytes and half a byte per plane
    (1, 12, 12, 256, 70, 3, 1, 1),   # 72 words: six panels of 12; 70 columns: the last output word is partly filled
    (1, 8, 6, 512, 64, 3, 1, 1),     # 144 words
    (1, 6, 6, 128, 33, 1, 1, 0),     # a 1x1 conv runs as a GEMM over the pixels: four words, one ragged panel
    (3, 7, 5, 640, 40, 1, 1, 0),     # twenty words: a panel of 16 and a ragged one
    (1, 5, 5, 128, 129, 5, 2, 2),    # 5x5 taps: 100 words, padding wider than one pixel, 129 columns
    (1, 11, 9, 256, 8, 3, 1, 0),     # eight columns: one wave across, no padding
    (2, 9, 10, 384, 24, 2, 1, 1),    # 2x2 taps of twelve words: 48 words, divisible by both panel lengths
    (1, 20, 20, 128, 16, 1, 2, 0),   # strided 1x1 (one tap): four words; 100 output rows
]


def panel_words(Kw, waves):
    """Panel length the kernel uses when `waves` waves share a reduction of Kw words (0: none): 12 when the
    reduction is whole 12-word panels and not whole 16-word ones, else 16; the other length only if it divides the
    reduction exactly; the number of panels must divide evenly over the waves."""
    first = 12 if Kw % 12 == 0 and Kw % 16 != 0 else 16
    second = 28 - first
    if -(-Kw // first) % waves == 0:
        return first
    if Kw % second == 0 and (Kw // second) % waves == 0:
        return second
    return 0


@pytest.mark.parametrize("shape", PANEL_KERNEL_SHAPES)
def test_conv_fused_panel_kernel_all_encodings(dlrt, oracle, shape):
    """tile_rows = 128 selects the kernel with one output row per lane that walks the reduction in panels against
    weights held in LDS; ksplit then is the number of 8-column groups a wave covers (1, 2 or 4; 0: 1).  Every output
    kind, and the packed-only call of a chained layer."""
    N, H, W, Ci, Co, k, stride, pad = shape
    cases = [(2, 2, UNSIGNED, TWOS, 2, (0, 1, 2)), (2, 1, UNSIGNED, BIPOLAR, 2, (1, 2, 4)), (1, 1, UNSIGNED, TWOS, 1, (1, 2, 4)),
             (1, 1, UNSIGNED, BIPOLAR, 4, (2, 4)), (2, 2, TWOS, UNSIGNED, 3, (1, 2)), (1, 4, UNSIGNED, TWOS, 2, (1, 2)),
             (4, 1, TWOS, TWOS, 2, (1, 2)), (1, 2, TWOS, TWOS, 2, (1, 4)), (3, 1, UNSIGNED, BIPOLAR, 2, (1, 2)),
             (2, 4, UNSIGNED, TWOS, 2, (1,)), (3, 2, UNSIGNED, TWOS, 2, (1,))]
    for idx, (abits, wbits, ea, ew, qbits, groups) in enumerate(cases):
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 38000 + idx + H)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 39000 + idx + Ci)
        for g in groups:
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=128, ksplit=g)
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=128, ksplit=g,
                       packed_only=True)
        # tile_rows = 128 s: s waves of a block share the tile's reduction, an equal number of panels each; a
        # split that no panel length (12 or 16 words) allows is refused
        Kw = k * k * ((Ci + 31) // 32)
        for s in (2, 3, 4):
            g = groups[-1]
            P = panel_words(Kw, s)
            # the block's weights over the padded reduction and the partial sums of the waves beyond the first
            lds = max(8 * max(g, 1) * wbits * (-(-Kw // P) * P if P else 0) * 4, (s - 1) * (8 * max(g, 1) * abits * wbits + abits) * 256)
            if P and lds <= 65536:
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=128 * s, ksplit=g)
                fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=128 * s, ksplit=g,
                           packed_only=True)
            else:
                with pytest.raises(dlrt.DlrtError):
                    fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=128 * s, ksplit=g)


def test_conv_fused_panel_kernel_rejects_what_it_cannot_hold(dlrt):
    def call(Ci, k, abits, wbits, ksplit=1):
        x = torch.zeros((1, 8, 8, Ci), dtype=torch.uint8, device=DEV)
        w = torch.zeros((16, k, k, Ci), dtype=torch.int8, device=DEV)
        X, Wp = dlrt.dlrt_pack_bitplanes(x, abits, UNSIGNED), dlrt.dlrt_pack_conv_weights(w, wbits, TWOS)
        s = torch.ones(16, device=DEV)
        dlrt.dlrt_bitserial_conv2d_fused(X, Wp, s, None, 1, 8, 8, Ci, 16, k, k, (1, 1), (k // 2, k // 2), abits, wbits, UNSIGNED,
                                         TWOS, qbits=2, out_q=torch.empty((1, 8, 8, 16), dtype=torch.uint8, device=DEV),
                                         tile_rows=128, ksplit=ksplit)
    call(128, 3, 2, 2)
    call(256, 1, 1, 4)
    for Ci, k, abits, wbits, ksplit in ((64, 3, 2, 2, 1),    # taps of two words
                                        (128, 3, 3, 3, 1),   # nine accumulators per column
                                        (128, 3, 2, 2, 4),   # thirty-two columns of four plane pairs
                                        (128, 3, 2, 2, 3)):  # no such column count
        with pytest.raises(dlrt.DlrtError):
            call(Ci, k, abits, wbits, ksplit)
    torch.cuda.synchronize()


def test_conv_fused_row_kernel_rejects_what_it_cannot_hold(dlrt):
    def call(Ci, k, pad):
        x = torch.zeros((1, 8, 8, Ci), dtype=torch.uint8, device=DEV)
        w = torch.zeros((16, k, k, Ci), dtype=torch.int8, device=DEV)
        X, Wp = dlrt.dlrt_pack_bitplanes(x, 2, UNSIGNED), dlrt.dlrt_pack_conv_weights(w, 2, TWOS)
        s = torch.ones(16, device=DEV)
        dlrt.dlrt_bitserial_conv2d_fused(X, Wp, s, None, 1, 8, 8, Ci, 16, k, k, (1, 1), (pad, pad), 2, 2, UNSIGNED, TWOS,
                                         qbits=2, out_q=torch.empty((1, 8 + 2 * pad - k + 1, 8 + 2 * pad - k + 1, 16),
                                                                    dtype=torch.uint8, device=DEV), tile_rows=64)
    call(64, 1, 0)  # two words: fits
    call(32, 3, 1)  # nine words: fits
    call(64, 3, 1)  # eighteen words (3x3 taps of two words): fits
    for Ci, k, pad in ((96, 3, 1), (544, 1, 0)):  # twenty-seven and seventeen words
        with pytest.raises(dlrt.DlrtError):
            call(Ci, k, pad)
    torch.cuda.synchronize()


def test_conv_fused_every_tile_height_and_reduction_split_gives_the_same_result(dlrt, oracle):
    """The tuning hints select the wave tile and how many waves split the reduction; all must agree."""
    x = inputs.uniform_values((1, 13, 11, 160), 2, UNSIGNED, 777)
    w = inputs.uniform_values((72, 3, 3, 160), 2, TWOS, 778)
    for tile_rows in (4, 8, 16, 32):  # 4: the half tile (two columns per lane) that narrow weights have besides the others
        for ksplit in (1, 2, 4, 8):
            fused_case(dlrt, oracle, x, w, 1, 1, 2, 2, UNSIGNED, TWOS, 2, tile_rows, ksplit)
            if tile_rows == 4:
                fused_case(dlrt, oracle, x, w, 1, 1, 2, 2, UNSIGNED, TWOS, 2, tile_rows, ksplit, packed_only=True)
    x4 = inputs.uniform_values((1, 9, 9, 96), 4, UNSIGNED, 779)
    w4 = inputs.uniform_values((40, 3, 3, 96), 4, TWOS, 780)
    for tile_rows in (4, 8):
        for ksplit in (1, 2, 4):  # 8 slices of a 4-bit x 4-bit tile would need more than 64 KB of LDS
            fused_case(dlrt, oracle, x4, w4, 2, 1, 4, 4, UNSIGNED, TWOS, 3, tile_rows, ksplit)
    xb = inputs.uniform_values((2, 6, 6, 64), 2, UNSIGNED, 781)
    wb = inputs.uniform_values((33, 3, 3, 64), 1, BIPOLAR, 782)
    for ksplit in (1, 2, 4):
        fused_case(dlrt, oracle, xb, wb, 1, 1, 2, 1, UNSIGNED, BIPOLAR, 2, 8, ksplit)
        fused_case(dlrt, oracle, xb, wb, 1, 1, 2, 1, UNSIGNED, BIPOLAR, 2, 4, ksplit)
    # few rows, many channels, a deep reduction: the planner's own choice is the half tile here
    xs = inputs.uniform_values((1, 7, 7, 256), 2, UNSIGNED, 783)
    ws = inputs.uniform_values((96, 3, 3, 256), 2, TWOS, 784)
    assert dlrt.dlrt_query_plan(49, 96, 9 * 256, 2, 2)["tile_rows"] == 4
    fused_case(dlrt, oracle, xs, ws, 1, 1, 2, 2, UNSIGNED, TWOS, 2)
    fused_case(dlrt, oracle, xs, ws, 1, 1, 2, 2, UNSIGNED, TWOS, 2, packed_only=True)
    x1 = inputs.uniform_values((1, 5, 5, 128), 1, UNSIGNED, 785)
    w1 = inputs.uniform_values((64, 3, 3, 128), 1, TWOS, 786)
    for ksplit in (1, 4):
        fused_case(dlrt, oracle, x1, w1, 1, 1, 1, 1, UNSIGNED, TWOS, 1, 4, ksplit)   # two accumulators per activation word


@pytest.mark.parametrize("widths", [(2, 1, BIPOLAR), (2, 2, TWOS), (1, 1, TWOS), (4, 4, TWOS)])
def test_conv_fused_pair_of_row_kernel_layers(dlrt, oracle, widths):
    """Two 1x1 convs on one image that both take the row kernel share a row-kernel launch when their reductions fill
    register rows of the same length: the YOLO-style split / merge pair (25600 pixels, 64 -> 32 and 64 -> 64 channels),
    a pair on different tensors with ragged shapes (32761 pixels x 40 channels over 100, 22500 x 96 over 128: rows of 4 words),
    and a pair whose rows differ in length, which goes out as two launches.  Packed output only, as in a chain, and
    every output kind."""
    abits, wbits, ew = widths
    cases = [((1, 160, 160, 64), 32, (1, 160, 160, 64), 64), ((1, 181, 181, 100), 40, (1, 150, 150, 128), 96),
             ((1, 80, 80, 128), 64, (1, 80, 80, 64), 64)]
    for idx, (xs0, co0, xs1, co1) in enumerate(cases):
        for packed_only in (True, False):
            probs, refs, keep = [], [], []
            for k, (xs, Co) in enumerate(((xs0, co0), (xs1, co1))):
                x = inputs.uniform_values(xs, abits, UNSIGNED, 63000 + 10 * idx + k)
                w = inputs.uniform_values((Co, 1, 1, xs[3]), wbits, ew, 64000 + 10 * idx + k)
                ref = oracle.conv2d_i32(x, w, (1, 1), (0, 0))
                scale, bias = calibrate(ref)
                y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=2)
                X = dlrt.dlrt_pack_bitplanes(src_tensor(x, UNSIGNED), abits, UNSIGNED)
                Wp = dlrt.dlrt_pack_conv_weights(src_tensor(w, ew), wbits, ew)
                Mo = ref.shape[0] * ref.shape[1] * ref.shape[2]
                acc = torch.full(ref.shape, -7, dtype=torch.int32, device=DEV)
                y = torch.full(ref.shape, -7.0, dtype=torch.float32, device=DEV)
                packed = torch.full((Mo, 2, (Co + 31) // 32), -1, dtype=torch.int32, device=DEV)
                sc, bs = dev(scale), dev(bias)
                probs.append(dlrt.conv_problem(X, Wp, sc, bs, xs[0], xs[1], xs[2], xs[3], Co, 1, 1, (1, 1), (0, 0), abits, wbits,
                                               qbits=2, out_acc=None if packed_only else acc, out_f32=None if packed_only else y,
                                               out_packed=packed))
                refs.append((ref, y_ref, oracle.pack_bitplanes(q_ref.reshape(Mo, Co).astype(np.int8), 2, UNSIGNED)))
                keep.append((X, Wp, sc, bs, acc, y, packed))
            dlrt.dlrt_bitserial_conv2d_fused_pair(probs[0], probs[1], abits, wbits, UNSIGNED, ew)
            torch.cuda.synchronize()
            for (ref, y_ref, p_ref), (_, _, _, _, acc, y, packed) in zip(refs, keep):
                assert np.array_equal(words(packed), p_ref), (idx, packed_only)
                if not packed_only:
                    assert np.array_equal(acc.cpu().numpy(), ref), idx
                    assert np.array_equal(y.cpu().numpy(), y_ref), idx


def test_conv_fused_pair_two_problems_in_one_launch(dlrt, oracle):
    """A stride-2 3x3 conv and the 1x1 stride-2 conv beside it (different reduction depths, so different
    numbers of waves would be planned), then two unrelated problems with ragged shapes; bipolar too."""
    cases = [((1, 28, 28, 128), (256, 3, 3, 128), 2, 1, (1, 28, 28, 128), (256, 1, 1, 128), 2, 0, 2, 2, TWOS),
             ((2, 9, 7, 40), (70, 3, 3, 40), 1, 1, (1, 12, 12, 96), (33, 1, 1, 96), 1, 0, 2, 2, TWOS),
             ((1, 20, 20, 256), (128, 1, 1, 256), 1, 0, (1, 20, 20, 256), (256, 1, 1, 256), 1, 0, 2, 1, BIPOLAR),
             ((1, 10, 10, 64), (16, 3, 3, 64), 1, 1, (1, 6, 6, 512), (40, 3, 3, 512), 1, 1, 4, 4, TWOS)]
    for idx, (xs0, ws0, st0, pd0, xs1, ws1, st1, pd1, abits, wbits, ew) in enumerate(cases):
        probs, refs, keep = [], [], []
        for k, (xs, ws, st, pd) in enumerate(((xs0, ws0, st0, pd0), (xs1, ws1, st1, pd1))):
            x = inputs.uniform_values(xs, abits, UNSIGNED, 61000 + 10 * idx + k)
            w = inputs.uniform_values(ws, wbits, ew, 62000 + 10 * idx + k)
            ref = oracle.conv2d_i32(x, w, (st, st), (pd, pd))
            scale, bias = calibrate(ref)
            y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=2)
            X = dlrt.dlrt_pack_bitplanes(src_tensor(x, UNSIGNED), abits, UNSIGNED)
            Wp = dlrt.dlrt_pack_conv_weights(src_tensor(w, ew), wbits, ew)
            Co, Mo = ws[0], ref.shape[0] * ref.shape[1] * ref.shape[2]
            acc = torch.full(ref.shape, -7, dtype=torch.int32, device=DEV)
            y = torch.full(ref.shape, -7.0, dtype=torch.float32, device=DEV)
            packed = torch.full((Mo, 2, (Co + 31) // 32), -1, dtype=torch.int32, device=DEV)
            sc, bs = dev(scale), dev(bias)
            probs.append(dlrt.conv_problem(X, Wp, sc, bs, xs[0], xs[1], xs[2], xs[3], Co, ws[1], ws[2], (st, st), (pd, pd),
                                           abits, wbits, qbits=2, out_acc=acc, out_f32=y, out_packed=packed))
            refs.append((ref, y_ref, oracle.pack_bitplanes(q_ref.reshape(Mo, Co).astype(np.int8), 2, UNSIGNED)))
            keep.append((X, Wp, sc, bs, acc, y, packed))
        dlrt.dlrt_bitserial_conv2d_fused_pair(probs[0], probs[1], abits, wbits, UNSIGNED, ew)
        torch.cuda.synchronize()
        for (ref, y_ref, p_ref), (_, _, _, _, acc, y, packed) in zip(refs, keep):
            assert np.array_equal(acc.cpu().numpy(), ref), idx
            assert np.array_equal(y.cpu().numpy(), y_ref), idx
            assert np.array_equal(words(packed), p_ref), idx


def test_conv_fused_rejects_hints_the_kernels_do_not_have(dlrt):
    X = torch.zeros((64, 4, 1), dtype=torch.int32, device=DEV)
    Wp = torch.zeros((8, 4, 9), dtype=torch.int32, device=DEV)
    acc = torch.zeros((1, 8, 8, 8), dtype=torch.int32, device=DEV)
    for tile_rows, ksplit in ((24, 0), (0, 3), (16, 0)):  # 16 rows needs too many accumulators at A4W4
        with pytest.raises(dlrt.DlrtError) as e:
            dlrt.dlrt_bitserial_conv2d_fused(X, Wp, None, None, 1, 8, 8, 32, 8, 3, 3, (1, 1), (1, 1), 4, 4, UNSIGNED,
                                             TWOS, out_acc=acc, tile_rows=tile_rows, ksplit=ksplit)
        assert e.value.code == 3


# ---- fused epilogue on the throughput (block) kernel: problems large enough to leave the per-wave kernel ----
@pytest.mark.parametrize("abits,wbits,ea,ew,qbits,M,N,K", [
    (2, 2, UNSIGNED, TWOS, 2, 1500, 1400, 200), (1, 1, UNSIGNED, BIPOLAR, 1, 2900, 2950, 608),
    (4, 4, UNSIGNED, TWOS, 4, 730, 750, 50), (3, 3, TWOS, TWOS, 3, 760, 710, 330), (2, 4, UNSIGNED, TWOS, 2, 1500, 700, 64)])
def test_gemm_fused_large_shapes(dlrt, oracle, abits, wbits, ea, ew, qbits, M, N, K):
    assert dlrt.dlrt_query_plan(M, N, K, abits, wbits)["kernel"] == "block"
    a = inputs.uniform_values((M, K), abits, ea, 41000 + M)
    w = inputs.uniform_values((N, K), wbits, ew, 42000 + N)
    ref = oracle.gemm_i32(a, w)  # every output against the oracle
    scale, bias = calibrate(ref)
    scale, bias = (scale * (1 << qbits) / 4).astype(np.float32), (bias * (1 << qbits) / 4).astype(np.float32)
    y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=qbits)
    A = dlrt.dlrt_pack_bitplanes(src_tensor(a, ea), abits, ea)
    W = dlrt.dlrt_pack_bitplanes(src_tensor(w, ew), wbits, ew)
    acc = torch.full((M, N), -7, dtype=torch.int32, device=DEV)
    y = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
    q = torch.full((M, N), 99, dtype=torch.uint8, device=DEV)
    packed = torch.full((M, qbits, (N + 31) // 32), -1, dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), dev(bias), M, N, K, abits, wbits, ea, ew, qbits=qbits, out_acc=acc,
                                   out_f32=y, out_q=q, out_packed=packed)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref)
    assert np.array_equal(y.cpu().numpy(), y_ref)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(words(packed), oracle.pack_bitplanes(q_ref.astype(np.int8), qbits, UNSIGNED))
    # only one output requested: the others stay untouched
    y2 = torch.empty((M, N), dtype=torch.float32, device=DEV)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), None, M, N, K, abits, wbits, ea, ew, out_f32=y2)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy(), oracle.epilogue_f32(ref, scale)[0])


def test_gemm_fused_small_shape_takes_the_per_wave_kernel(dlrt, oracle):
    c, a, w = inputs.config1()
    ref = oracle.gemm_i32(a, w)
    scale = inputs.uniform_scale(c.N, 5)
    A = dlrt.dlrt_pack_bitplanes(src_tensor(a, c.enc_a), 2, c.enc_a)
    W = dlrt.dlrt_pack_bitplanes(src_tensor(w, c.enc_w), 2, c.enc_w)
    y = torch.empty((c.M, c.N), dtype=torch.float32, device=DEV)
    packed = torch.empty((c.M, 2, 2), dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), None, c.M, c.N, c.K, 2, 2, c.enc_a, c.enc_w, out_f32=y, out_packed=packed)
    torch.cuda.synchronize()
    y_ref, q_ref = oracle.epilogue_f32(ref, scale, qbits=2)
    assert np.array_equal(y.cpu().numpy(), y_ref)
    assert np.array_equal(words(packed), oracle.pack_bitplanes(q_ref.astype(np.int8), 2, UNSIGNED))


@pytest.mark.parametrize("abits,wbits,ea,ew,qbits,M,N,K", [
    (2, 2, UNSIGNED, TWOS, 2, 20000, 40, 50), (2, 1, UNSIGNED, BIPOLAR, 2, 100000, 33, 200),
    (4, 4, TWOS, TWOS, 4, 200000, 7, 256), (1, 3, UNSIGNED, UNSIGNED, 1, 70001, 64, 31), (3, 2, TWOS, UNSIGNED, 3, 33000, 128, 64),
    (2, 2, UNSIGNED, TWOS, 2, 10000, 300, 288), (2, 2, UNSIGNED, TWOS, 2, 60000, 130, 576), (1, 1, UNSIGNED, BIPOLAR, 2, 100100, 256, 500)])
def test_gemm_tall_skinny_takes_the_row_kernel(dlrt, oracle, abits, wbits, ea, ew, qbits, M, N, K):
    """A reduction of at most 16 words (or 18) and enough waves of 64 rows x 32 columns: the planner picks the
    kernel with one output row per lane, for the plain GEMM and for every output of the fused one."""
    assert dlrt.dlrt_query_plan(M, N, K, abits, wbits)["kernel"] == "rows"
    a = inputs.uniform_values((M, K), abits, ea, 41000 + M % 97)
    w = inputs.uniform_values((N, K), wbits, ew, 42000 + N)
    ref = oracle.gemm_i32(a, w)
    assert np.array_equal(gpu_gemm(dlrt, a, w, abits, wbits, ea, ew), ref)
    scale, bias = calibrate(ref)
    scale, bias = (scale * (1 << qbits) / 4).astype(np.float32), (bias * (1 << qbits) / 4).astype(np.float32)
    y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=qbits)
    want = oracle.pack_bitplanes(q_ref.astype(np.int8), qbits, UNSIGNED)
    A = dlrt.dlrt_pack_bitplanes(src_tensor(a, ea), abits, ea)
    W = dlrt.dlrt_pack_bitplanes(src_tensor(w, ew), wbits, ew)
    acc = torch.full((M, N), -7, dtype=torch.int32, device=DEV)
    y = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
    q = torch.full((M, N), 99, dtype=torch.uint8, device=DEV)
    packed = torch.full((M, qbits, (N + 31) // 32), -1, dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), dev(bias), M, N, K, abits, wbits, ea, ew, qbits=qbits, out_acc=acc,
                                   out_f32=y, out_q=q, out_packed=packed)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref)
    assert np.array_equal(y.cpu().numpy(), y_ref)
    assert np.array_equal(q.cpu().numpy(), q_ref)
    assert np.array_equal(words(packed), want)
    packed.fill_(-1)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), None, M, N, K, abits, wbits, ea, ew, qbits=qbits, out_packed=packed)
    torch.cuda.synchronize()
    _, q_nobias = oracle.epilogue_f32(ref, scale, None, qbits=qbits)
    assert np.array_equal(words(packed), oracle.pack_bitplanes(q_nobias.astype(np.int8), qbits, UNSIGNED))


def test_random_gemms_across_the_kernel_choice_boundaries(dlrt, oracle):
    """Seeded random shapes, bit widths and encodings, drawn around the sizes where the planner switches
    between the row, per-wave and block kernels; every output of the fused GEMM against the oracle."""
    r = np.random.default_rng(20220708)
    kinds = set()
    for case in range(48):
        abits, wbits = int(r.integers(1, 5)), int(r.integers(1, 5))
        ea = int(r.choice([UNSIGNED, TWOS]))
        ew = BIPOLAR if wbits == 1 and r.random() < 0.5 else int(r.choice([UNSIGNED, TWOS]))
        M = int(r.choice([1, 63, 64, 65, 1000, 2047, 2048, 2049, 16384, 16385, 40000, 65535, 65536, 70000]))
        N = int(r.choice([1, 31, 32, 33, 64, 65, 96, 128, 200, 288]))
        K = int(r.choice([1, 31, 32, 33, 64, 65, 128, 256, 257, 288, 289, 512, 513, 544, 570, 576, 600]))
        if M * N * K > 3e9:   # keep the oracle's share of the test short
            M = 16385
        qbits = int(r.integers(1, 5))
        kinds.add(dlrt.dlrt_query_plan(M, N, K, abits, wbits)["kernel"])
        a = inputs.uniform_values((M, K), abits, ea, 51000 + case)
        w = inputs.uniform_values((N, K), wbits, ew, 52000 + case)
        ref = oracle.gemm_i32(a, w)
        scale, bias = calibrate(ref)
        scale, bias = (scale * (1 << qbits) / 4).astype(np.float32), (bias * (1 << qbits) / 4).astype(np.float32)
        y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=qbits)
        A = dlrt.dlrt_pack_bitplanes(src_tensor(a, ea), abits, ea)
        W = dlrt.dlrt_pack_bitplanes(src_tensor(w, ew), wbits, ew)
        acc = torch.full((M, N), -7, dtype=torch.int32, device=DEV)
        y = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
        packed = torch.full((M, qbits, (N + 31) // 32), -1, dtype=torch.int32, device=DEV)
        dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), dev(bias), M, N, K, abits, wbits, ea, ew, qbits=qbits,
                                       out_acc=acc, out_f32=y)
        dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), dev(bias), M, N, K, abits, wbits, ea, ew, qbits=qbits,
                                       out_packed=packed)
        torch.cuda.synchronize()
        tag = (case, M, N, K, abits, wbits, ea, ew, qbits)
        assert np.array_equal(acc.cpu().numpy(), ref), tag
        assert np.array_equal(y.cpu().numpy(), y_ref), tag
        assert np.array_equal(words(packed), oracle.pack_bitplanes(q_ref.astype(np.int8), qbits, UNSIGNED)), tag
    assert kinds == {"rows", "wave", "block"}


def test_random_convs_across_the_kernel_choice_boundaries(dlrt, oracle):
    """The same for convolutions: kernel size, stride, padding, batch and channel counts drawn so that all
    three kernels and ragged words / tiles occur; all four outputs, then the packed-only call."""
    r = np.random.default_rng(8820)
    kinds = set()
    for case in range(40):
        abits, wbits = int(r.integers(1, 5)), int(r.integers(1, 5))
        ea = int(r.choice([UNSIGNED, TWOS]))
        ew = BIPOLAR if wbits == 1 and r.random() < 0.5 else int(r.choice([UNSIGNED, TWOS]))
        k = int(r.choice([1, 1, 2, 3, 3, 5]))
        stride, pad = int(r.choice([1, 1, 2])), int(r.choice([0, 1, k // 2]))
        Ci = int(r.choice([3, 16, 32, 33, 64, 100, 256]))
        Co = int(r.choice([1, 8, 32, 40, 64, 130]))
        H, W_ = int(r.choice([5, 40, 130, 130])), int(r.choice([7, 128, 128]))
        N = int(r.choice([1, 5, 5]))
        Ho, Wo = (H + 2 * pad - k) // stride + 1, (W_ + 2 * pad - k) // stride + 1
        if Ho <= 0 or Wo <= 0:
            continue
        if N * Ho * Wo * Co * k * k * Ci > 2.5e9:
            N, Ci = 1, min(Ci, 33)
        qbits = int(r.integers(1, 5))
        kinds.add(dlrt.dlrt_query_plan(N * Ho * Wo, Co, k * k * ((Ci + 31) // 32) * 32, abits, wbits)["kernel"])
        x = inputs.uniform_values((N, H, W_, Ci), abits, ea, 61000 + case)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 62000 + case)
        fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits)
        fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, packed_only=True)
    assert kinds == {"rows", "wave", "block"}


def test_conv_fused_large_batch_takes_the_block_kernel(dlrt, oracle):
    """Batch 16 of the 56 x 56 x 64 layer: 784 block tiles, so the throughput kernel runs the fused epilogue."""
    x = inputs.uniform_values((16, 56, 56, 64), 2, UNSIGNED, 888)
    w = inputs.uniform_values((64, 3, 3, 64), 2, TWOS, 889)
    fused_case(dlrt, oracle, x, w, 1, 1, 2, 2, UNSIGNED, TWOS, 2)
    xb = inputs.uniform_values((9, 40, 40, 96), 2, UNSIGNED, 890)
    wb = inputs.uniform_values((160, 3, 3, 96), 1, BIPOLAR, 891)
    fused_case(dlrt, oracle, xb, wb, 2, 1, 2, 1, UNSIGNED, BIPOLAR, 2)


# ---- streams: every call enqueues on the stream it is given and never synchronises -------------------------
def test_calls_follow_the_current_stream_and_two_streams_do_not_mix(dlrt, oracle):
    """Two independent pack -> GEMM -> epilogue chains, each enqueued on a stream of its own (the binding hands
    torch's current stream to the C ABI), interleaved call by call; results are read only after each stream's
    own synchronisation."""
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    cases = [(300, 200, 1000, 2, 2, TWOS), (257, 129, 4100, 4, 1, BIPOLAR)]
    host, state = [], [{}, {}]
    for i, (M, N, K, abits, wbits, ew) in enumerate(cases):
        a = inputs.uniform_values((M, K), abits, UNSIGNED, 57000 + i)
        w = inputs.uniform_values((N, K), wbits, ew, 57010 + i)
        host.append((a, w, inputs.uniform_scale(N, 57020 + i)))
    steps = ["upload", "pack_a", "pack_w", "gemm", "epilogue"]
    for step in steps:  # interleave the two chains step by step
        for i, (M, N, K, abits, wbits, ew) in enumerate(cases):
            st, (a, w, scale) = state[i], host[i]
            with torch.cuda.stream(streams[i]):
                if step == "upload":
                    st["a"], st["w"], st["s"] = src_tensor(a, UNSIGNED), src_tensor(w, ew), dev(scale)
                elif step == "pack_a":
                    st["A"] = dlrt.dlrt_pack_bitplanes(st["a"], abits, UNSIGNED)
                elif step == "pack_w":
                    st["W"] = dlrt.dlrt_pack_bitplanes(st["w"], wbits, ew)
                elif step == "gemm":
                    st["C"] = dlrt.dlrt_bitserial_gemm(st["A"], st["W"], M, N, K, abits, wbits, UNSIGNED, ew)
                else:
                    st["y"], st["q"] = dlrt.dlrt_epilogue_f32(st["C"], st["s"], qbits=2)
    for i, (M, N, K, abits, wbits, ew) in enumerate(cases):
        streams[i].synchronize()
        a, w, scale = host[i]
        ref = oracle.gemm_i32(a, w)
        y_ref, q_ref = oracle.epilogue_f32(ref, scale, qbits=2)
        assert np.array_equal(state[i]["C"].cpu().numpy(), ref), i
        assert np.array_equal(state[i]["y"].cpu().numpy(), y_ref) and np.array_equal(state[i]["q"].cpu().numpy(), q_ref), i
    torch.cuda.synchronize()


# ---- sizes at the far ends -------------------------------------------------------------------------------
def test_gemm_very_tall_output_indexing_beyond_2_31_bytes(dlrt, oracle):
    """M = 2^24 + 5 rows of 40 outputs: the int32 result is 2.7 GB, so byte offsets pass 2^31; sampled rows
    against the oracle plus the column-sum identity over everything."""
    M, N, K = (1 << 24) + 5, 40, 64
    a = inputs.uniform_values((M, K), 2, UNSIGNED, 51000)
    w = inputs.uniform_values((N, K), 2, TWOS, 51001)
    A = dlrt.dlrt_pack_bitplanes(dev(a.astype(np.uint8)), 2, UNSIGNED)
    W = dlrt.dlrt_pack_bitplanes(dev(w), 2, TWOS)
    C = dlrt.dlrt_bitserial_gemm(A, W, M, N, K, 2, 2, UNSIGNED, TWOS)
    torch.cuda.synchronize()
    rows = np.concatenate([rng(5).choice(M, size=64, replace=False), [0, M - 1, (1 << 23) + 1]])
    assert np.array_equal(C[torch.as_tensor(rows, device=DEV)].cpu().numpy(), oracle.gemm_i32(a[rows], w))
    colsum = C.sum(dim=0, dtype=torch.int64).cpu().numpy()
    assert np.array_equal(colsum, w.astype(np.int64) @ a.sum(axis=0, dtype=np.int64))


def every_output_agrees(acc, y, q, packed, scale, bias, qbits, chunk=1 << 16):
    """Whole-tensor consistency of the four fused outputs, evaluated on the GPU with torch in row chunks:
    y against float64 acc * scale + bias rounded to fp32 (at most 1 ulp off a fused multiply-add), q against
    clamp(rint(y)), packed against the bits of q.  The absolute values are pinned by the sampled rows."""
    M, N = acc.shape
    sc, bs = dev(scale).double(), dev(bias).double()
    shifts = torch.arange(32, device=DEV, dtype=torch.int64)
    for r0 in range(0, M, chunk):
        a, yy, qq = acc[r0:r0 + chunk], y[r0:r0 + chunk], q[r0:r0 + chunk]
        want = (a.double() * sc + bs).float()
        ulp = torch.maximum(want.abs(), torch.tensor(1e-30, device=DEV)) * 2.0 ** -23
        assert bool(((yy - want).abs() <= ulp).all()), r0
        assert torch.equal(qq, torch.clamp(torch.round(yy), 0, (1 << qbits) - 1).to(torch.uint8)), r0
        pad = (-N) % 32
        bits = torch.nn.functional.pad(qq, (0, pad)).to(torch.int64).reshape(qq.shape[0], -1, 32)
        for p in range(qbits):
            word = (((bits >> p) & 1) << shifts).sum(dim=2)
            got = packed[r0:r0 + chunk, p].to(torch.int64) & 0xFFFFFFFF
            assert torch.equal(got, word), (r0, p)


@pytest.mark.parametrize("kernel,M,N,K,abits,wbits,ew", [
    ("block", 1040013, 2080, 680, 2, 2, TWOS),         # 2.16e9 outputs, ragged in M, N and K (22 words)
    ("rows", (1 << 25) + 21, 65, 32, 2, 1, BIPOLAR)])  # 2.18e9 outputs, one word per row
def test_gemm_more_than_2_31_outputs(dlrt, oracle, kernel, M, N, K, abits, wbits, ew):
    """Element indices of every output pass 2^31 (an int32 result of 8.7 GB): sampled rows of all four fused
    outputs against the oracle (first, last, the rows either side of element 2^31, random ones), the
    column-sum identity over all accumulators, and the other outputs against the accumulators everywhere."""
    assert M * N > 1 << 31 and dlrt.dlrt_query_plan(M, N, K, abits, wbits)["kernel"] == kernel
    qbits = 2
    a = inputs.uniform_values((M, K), abits, UNSIGNED, 54000 + N)
    w = inputs.uniform_values((N, K), wbits, ew, 54001 + N)
    edge = (1 << 31) // N
    rows = np.concatenate([rng(N).choice(M, size=256, replace=False), [0, M - 1, edge - 1, edge, edge + 1]])
    ref = oracle.gemm_i32(a[rows], w)
    scale, bias = calibrate(ref)
    y_ref, q_ref = oracle.epilogue_f32(ref, scale, bias, qbits=qbits)
    A = dlrt.dlrt_pack_bitplanes(dev(a.astype(np.uint8)), abits, UNSIGNED)
    W = dlrt.dlrt_pack_bitplanes(src_tensor(w, ew), wbits, ew)
    acc = torch.full((M, N), -7, dtype=torch.int32, device=DEV)
    y = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
    q = torch.full((M, N), 99, dtype=torch.uint8, device=DEV)
    packed = torch.full((M, qbits, (N + 31) // 32), -1, dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_gemm_fused(A, W, dev(scale), dev(bias), M, N, K, abits, wbits, UNSIGNED, ew, qbits=qbits,
                                   out_acc=acc, out_f32=y, out_q=q, out_packed=packed)
    torch.cuda.synchronize()
    pick = torch.as_tensor(rows, device=DEV)
    assert np.array_equal(acc[pick].cpu().numpy(), ref)
    assert np.array_equal(y[pick].cpu().numpy(), y_ref)
    assert np.array_equal(q[pick].cpu().numpy(), q_ref)
    assert np.array_equal(words(packed[pick]), oracle.pack_bitplanes(q_ref.astype(np.int8), qbits, UNSIGNED))
    colsum = acc.sum(dim=0, dtype=torch.int64).cpu().numpy()
    assert np.array_equal(colsum, w.astype(np.int64) @ a.sum(axis=0, dtype=np.int64))
    every_output_agrees(acc, y, q, packed, scale, bias, qbits)
    # the plain call writes the same accumulators
    plain = dlrt.dlrt_bitserial_gemm(A, W, M, N, K, abits, wbits, UNSIGNED, ew)
    torch.cuda.synchronize()
    assert torch.equal(plain, acc)


@pytest.mark.parametrize("kernel,Ci,Co,k,hint", [("rows", 32, 32, 3, 0), ("block", 96, 40, 3, 0), ("wave", 32, 24, 1, 8)])
def test_conv_image_too_large_for_multiply_high_division(dlrt, oracle, kernel, Ci, Co, k, hint):
    """2048 x 2048 output pixels: pixels * width passes 2^32, so output row -> (image, row, column) uses the
    hardware's division instead of the multiply-high shortcut, in each of the three kernels."""
    H = W = 2048
    if not hint:
        assert dlrt.dlrt_query_plan(H * W, Co, k * k * (Ci // 32) * 32, 2, 2)["kernel"] == kernel
    x = inputs.uniform_values((1, H, W, Ci), 2, UNSIGNED, 55000 + Co)
    w = inputs.uniform_values((Co, k, k, Ci), 2, TWOS, 55001 + Co)
    ref = oracle.conv2d_i32(x, w, (1, 1), (k // 2, k // 2))
    X = dlrt.dlrt_pack_bitplanes(src_tensor(x, UNSIGNED), 2, UNSIGNED)
    Wp = dlrt.dlrt_pack_conv_weights(dev(w), 2, TWOS)
    acc = torch.full((1, H, W, Co), -7, dtype=torch.int32, device=DEV)
    dlrt.dlrt_bitserial_conv2d_fused(X, Wp, None, None, 1, H, W, Ci, Co, k, k, (1, 1), (k // 2, k // 2), 2, 2, UNSIGNED,
                                     TWOS, out_acc=acc, tile_rows=hint)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), ref)


def test_pack_and_epilogue_more_than_2_31_elements(dlrt, oracle):
    """The two streaming kernels past 2^31 elements.  Pack: 70001 x 32040 uint8 (2.24e9 values, ragged last
    word, rows of 1002 words), sampled rows against the oracle and every plane's popcount against a count of
    the values that have the bit.  Epilogue: 1100003 x 2000 accumulators (8.8 GB) drawn on the GPU, sampled
    rows against the oracle and requantized output against the fp32 output everywhere."""
    rows, K = 70001, 32040
    q = inputs.uniform_values((rows, K), 2, UNSIGNED, 56000).astype(np.uint8)
    packed = dlrt.dlrt_pack_bitplanes(dev(q), 2, UNSIGNED)
    torch.cuda.synchronize()
    edge = (1 << 31) // K
    pick = np.concatenate([rng(56).choice(rows, size=128, replace=False), [0, rows - 1, edge - 1, edge, edge + 1]])
    assert np.array_equal(words(packed[torch.as_tensor(pick, device=DEV)]), oracle.pack_bitplanes(q[pick].astype(np.int8), 2, UNSIGNED))
    ones = torch.zeros(2, dtype=torch.int64, device=DEV)
    table = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=DEV)
    for r0 in range(0, rows, 4096):  # popcount per plane by bytes through a 256-entry table
        part = packed[r0:r0 + 4096].contiguous().view(torch.uint8).reshape(-1, 2, 4 * packed.shape[2])
        ones += table[part.long()].sum(dim=(0, 2))
    assert ones.tolist() == [int(np.count_nonzero(q & 1)), int(np.count_nonzero(q & 2))]
    del packed, q

    M, C = 1100003, 2000
    gen = torch.Generator(device=DEV).manual_seed(56001)
    acc = torch.randint(-40000, 40000, (M, C), dtype=torch.int32, device=DEV, generator=gen)
    scale = inputs.uniform_scale(C, 56002, 2e-5, 6e-5)
    bias = inputs.uniform_scale(C, 56003, 1.0, 2.0)
    y, qq = dlrt.dlrt_epilogue_f32(acc, dev(scale), dev(bias), qbits=2)
    torch.cuda.synchronize()
    edge = (1 << 31) // C
    pick = torch.as_tensor(np.concatenate([rng(57).choice(M, size=128, replace=False), [0, M - 1, edge - 1, edge, edge + 1]]), device=DEV)
    y_ref, q_ref = oracle.epilogue_f32(acc[pick].cpu().numpy(), scale, bias, qbits=2)
    assert np.array_equal(y[pick].cpu().numpy(), y_ref) and np.array_equal(qq[pick].cpu().numpy(), q_ref)
    assert len(np.unique(q_ref)) == 4
    sc, bs = dev(scale).double(), dev(bias).double()
    for r0 in range(0, M, 1 << 16):
        want = (acc[r0:r0 + (1 << 16)].double() * sc + bs).float()
        got = y[r0:r0 + (1 << 16)]
        assert bool(((got - want).abs() <= want.abs() * 2.0 ** -23).all()), r0
        assert torch.equal(qq[r0:r0 + (1 << 16)], torch.clamp(torch.round(got), 0, 3).to(torch.uint8)), r0


def test_gemm_very_long_reduction(dlrt, oracle):
    """K = 2^20 + 37 (32769 words per plane, ragged last word), small M and N: many chunks per wave."""
    M, N, K = 20, 70, (1 << 20) + 37
    for abits, wbits, ew in ((2, 2, TWOS), (1, 1, BIPOLAR), (4, 4, TWOS)):
        a = inputs.uniform_values((M, K), abits, UNSIGNED, 52000 + abits)
        w = inputs.uniform_values((N, K), wbits, ew, 52100 + wbits)
        assert np.array_equal(gpu_gemm(dlrt, a, w, abits, wbits, UNSIGNED, ew), oracle.gemm_i32(a, w))


def test_conv_large_image_single_channel_word(dlrt, oracle):
    """640 x 640 x 32 input (the YOLO-style stem size), 3x3 stride 2: 102400 output pixels, one word per pixel."""
    x = inputs.uniform_values((1, 640, 640, 32), 2, UNSIGNED, 53000)
    w = inputs.uniform_values((32, 3, 3, 32), 1, BIPOLAR, 53001)
    got = gpu_conv(dlrt, x, w, (2, 2), (1, 1), 2, 1, UNSIGNED, BIPOLAR)
    assert np.array_equal(got, oracle.conv2d_i32(x, w, (2, 2), (1, 1)))


# ---- GEMM through both kernels: large shapes take the block kernel, small ones the per-wave kernel ----
def test_gemm_ragged_large_shape_block_kernel(dlrt, oracle):
    for abits, wbits, ea, ew, M, N, K in [(2, 2, UNSIGNED, TWOS, 1500, 1400, 200), (1, 1, UNSIGNED, BIPOLAR, 2900, 2950, 608),
                                          (4, 4, UNSIGNED, TWOS, 730, 750, 50), (3, 3, TWOS, TWOS, 760, 710, 330),
                                          (1, 1, UNSIGNED, TWOS, 3000, 2900, 530)]:
        assert dlrt.dlrt_query_plan(M, N, K, abits, wbits)["kernel"] == "block"
        a = inputs.uniform_values((M, K), abits, ea, 31000 + M)
        w = inputs.uniform_values((N, K), wbits, ew, 32000 + N)
        got = gpu_gemm(dlrt, a, w, abits, wbits, ea, ew)
        assert np.array_equal(got, oracle.gemm_i32(a, w)), (abits, wbits)  # every output against the oracle


# ---- comparison variant: int8 matrix-instruction GEMM on the unpacked values ----------------------------
@pytest.mark.parametrize("M,N,K", [(128, 128, 128), (1, 1, 16), (200, 300, 208), (130, 70, 1040), (512, 512, 512)])
def test_unpacked_gemm_i8_matches_oracle(dlrt, oracle, M, N, K):
    r = rng(M * 7 + N)
    for lo, hi in ((0, 4), (-2, 2), (-8, 16), (-128, 128)):
        a = r.integers(lo, hi, size=(M, K)).astype(np.int8)
        w = r.integers(lo, hi, size=(N, K)).astype(np.int8)
        got = dlrt.dlrt_unpacked_gemm_i8(dev(a), dev(w))
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.gemm_i32(a, w)), (lo, hi)


def test_unpacked_gemm_i8_agrees_with_the_bit_serial_gemm_at_full_size(dlrt, oracle):
    c, a, w = inputs.config5(2, 2)
    got = dlrt.dlrt_unpacked_gemm_i8(dev(a.astype(np.int8)), dev(w))
    ref = gpu_gemm(dlrt, a, w, 2, 2, c.enc_a, c.enc_w)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    rows = rng(56).choice(c.M, size=32, replace=False)
    assert np.array_equal(got[rows], oracle.gemm_i32(a[rows], w))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("M,N,K", [(128, 128, 256), (1, 1, 32), (200, 300, 224), (130, 70, 1056), (257, 129, 4096)])
def test_unpacked_gemm_i4_matches_oracle(dlrt, oracle, M, N, K):
    """The 8-way dot-product variant on signed 4-bit values: every value of [-8, 7] on both sides, ragged tiles,
    reductions that are not whole 256-element chunks."""
    r = rng(M * 11 + N)
    a = r.integers(-8, 8, size=(M, K)).astype(np.int8)
    w = r.integers(-8, 8, size=(N, K)).astype(np.int8)
    A4, W4 = dlrt.dlrt_pack_nibbles(dev(a)), dlrt.dlrt_pack_nibbles(dev(w))
    got = dlrt.dlrt_unpacked_gemm_i4(A4, W4, K)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.gemm_i32(a, w))


def test_unpacked_gemm_i4_agrees_with_the_bit_serial_gemm_at_full_size(dlrt, oracle):
    c, a, w = inputs.config5(2, 2)
    got = dlrt.dlrt_unpacked_gemm_i4(dlrt.dlrt_pack_nibbles(dev(a.astype(np.int8))), dlrt.dlrt_pack_nibbles(dev(w)), c.K)
    ref = gpu_gemm(dlrt, a, w, 2, 2, c.enc_a, c.enc_w)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    rows = rng(57).choice(c.M, size=32, replace=False)
    assert np.array_equal(got[rows], oracle.gemm_i32(a[rows], w))
    assert np.array_equal(got, ref)


# ---- seeded random shapes, encodings and kernel hints ---------------------------------------------------------
@pytest.mark.parametrize("seed", [101, 102, 103])
def test_random_convs_planned_and_hinted_match_the_oracle(dlrt, oracle, seed):
    """Random small convolutions over every bit width and encoding: the planned kernel with every kind of output,
    and the chained-layer call (packed output only) under a random row- or panel-kernel hint; a hint the kernels
    do not have must be refused, any other must give the oracle's words."""
    r = rng(seed)
    ran = refused = 0
    for case in range(60):
        abits, wbits, qbits = int(r.integers(1, 5)), int(r.integers(1, 5)), int(r.integers(1, 5))
        ea = int(r.choice([UNSIGNED, UNSIGNED, TWOS]))
        ew = BIPOLAR if wbits == 1 and r.random() < 0.5 else int(r.choice([UNSIGNED, TWOS]))
        k = int(r.choice([1, 3, 3]))
        stride, pad = int(r.choice([1, 1, 2])), k // 2
        panel = r.random() < 0.5
        if panel:   # whole 16-byte groups per tap
            Ci, Co = int(r.choice([128, 256, 384, 512])), int(r.choice([8, 24, 32, 64, 72, 128]))
            hint = (128 * int(r.integers(1, 5)), int(r.choice([1, 1, 2, 4])))
        else:       # at most 18 reduction words
            Ci, Co = int(r.choice([16, 32, 64, 100, 128] if k == 1 else [16, 32, 64])), int(r.choice([32, 64, 96, 128, 40]))
            hint = (64, int(r.choice([1, 2, 4, 8, 12])))
        H, W, N = int(r.choice([6, 20, 33])), int(r.choice([7, 24, 40])), int(r.choice([1, 2, 5]))
        x = inputs.uniform_values((N, H, W, Ci), abits, ea, 50000 + 100 * seed + case)
        w = inputs.uniform_values((Co, k, k, Ci), wbits, ew, 60000 + 100 * seed + case)
        if case % 3 == 0:
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits)
        try:
            fused_case(dlrt, oracle, x, w, stride, pad, abits, wbits, ea, ew, qbits, tile_rows=hint[0], ksplit=hint[1],
                       packed_only=True)
            ran += 1
        except dlrt.DlrtError as e:
            assert e.code == 3, (case, hint)   # a shape / hint the kernel does not have: nothing was launched
            refused += 1
    assert ran >= 20 and refused >= 5, (ran, refused)


# ---- error handling with real buffers ------------------------------------------------------------------
def test_errors_raise_and_launch_nothing(dlrt):
    a = torch.zeros((4, 2, 1), dtype=torch.int32, device=DEV)
    out = torch.full((4, 4), 77, dtype=torch.int32, device=DEV)
    with pytest.raises(dlrt.DlrtError) as e:
        dlrt.dlrt_bitserial_gemm(a, a, 4, 4, 32, 2, 2, BIPOLAR, TWOS, out=out)
    assert e.value.code == 4
    wide = torch.zeros((4, 7, 1), dtype=torch.int32, device=DEV)  # large enough for the binding's own size check
    with pytest.raises(dlrt.DlrtError) as e:
        dlrt.dlrt_bitserial_gemm(a, wide, 4, 4, 32, 2, 7, UNSIGNED, TWOS, out=out)
    assert e.value.code == 2
    with pytest.raises(ValueError):  # a weight buffer packed for fewer bits than the call names never reaches the library
        dlrt.dlrt_bitserial_gemm(a, a, 4, 4, 32, 2, 4, UNSIGNED, TWOS, out=out)
    torch.cuda.synchronize()
    assert torch.all(out == 77)
