"""Pins for the CPU oracle's layer primitives: library routines (torch CPU, float64 -- exact
for these small integers), closed forms, brute force and exact rational arithmetic."""
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

RNG = np.random.default_rng(20220913)


def rand_i8(*shape, lo=-128, hi=127):
    return RNG.integers(lo, hi + 1, size=shape, dtype=np.int64).astype(np.int8)


def torch_conv(x, w, bias, stride, pad, groups=1):
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)           # [co][ci][kh][kw]
    bt = None if bias is None else torch.from_numpy(bias.astype(np.float64))
    y = F.conv2d(xt, wt, bt, stride=stride, padding=pad, groups=groups)
    return y.permute(0, 2, 3, 1).numpy()


CONV_CASES = [  # n, h, w, ci, co, k, stride, pad
    (2, 5, 7, 3, 4, 3, 1, 1), (1, 8, 8, 16, 8, 3, 2, 1), (2, 9, 6, 5, 7, 1, 1, 0), (1, 7, 7, 4, 6, 1, 2, 0),
    (1, 11, 13, 3, 5, 7, 2, 3), (3, 4, 4, 2, 3, 3, 2, 1), (1, 6, 5, 8, 8, 5, 1, 2), (1, 3, 3, 1, 1, 3, 1, 0),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_library_conv_and_toeplitz(orc, case):
    n, h, w, ci, co, k, stride, pad = case
    x, wt = rand_i8(n, h, w, ci), rand_i8(co, k, k, ci)
    bias = RNG.integers(-5000, 5000, size=co).astype(np.int32)
    acc = orc.conv_acc_i8(x, wt, bias, stride, pad)
    ref = torch_conv(x, wt, bias, stride, pad)
    assert acc.shape == ref.shape
    assert np.array_equal(acc.astype(np.float64), ref)
    assert np.array_equal(acc, orc.conv_acc_i8(x, wt, bias, stride, pad, toeplitz=True))


RECT_CASES = [  # n, h, w, ci, co, kh, kw, stride, pad (rows), pad_w (columns): kernels that are not square
    (2, 6, 9, 3, 4, 1, 7, 1, 0, 3), (1, 9, 6, 5, 3, 7, 1, 1, 3, 0), (2, 5, 5, 4, 4, 1, 3, 1, 0, 1), (1, 5, 5, 4, 6, 3, 1, 1, 1, 0),
    (1, 8, 10, 2, 3, 3, 5, 2, 1, 2), (1, 7, 7, 3, 2, 5, 5, 1, 2, 2), (1, 9, 9, 2, 2, 3, 3, 2, 0, 0),
]


@pytest.mark.parametrize("case", RECT_CASES)
def test_rectangular_kernels_and_per_axis_padding(orc, case):
    """Against the library convolution, against the second (Toeplitz) formulation, and against the transposed problem:
    swapping the image axes, the kernel axes and the two paddings must give the transposed result."""
    n, h, w, ci, co, kh, kw, stride, pad, pad_w = case
    x, wt = rand_i8(n, h, w, ci), rand_i8(co, kh, kw, ci)
    bias = RNG.integers(-5000, 5000, size=co).astype(np.int32)
    acc = orc.conv_acc_i8(x, wt, bias, stride, pad, pad_w=pad_w)
    ref = torch_conv(x, wt, bias, stride, (pad, pad_w))
    assert acc.shape == ref.shape and np.array_equal(acc.astype(np.float64), ref)
    assert np.array_equal(acc, orc.conv_acc_i8(x, wt, bias, stride, pad, toeplitz=True, pad_w=pad_w))
    swapped = orc.conv_acc_i8(np.ascontiguousarray(x.transpose(0, 2, 1, 3)), np.ascontiguousarray(wt.transpose(0, 2, 1, 3)), bias, stride, pad_w, pad_w=pad)
    assert np.array_equal(acc, swapped.transpose(0, 2, 1, 3))


def test_row_kernel_counts_in_range_taps(orc):
    """All-ones 1x7 kernel with 3 columns of padding on an all-ones row of 9: 4 5 6 7 7 7 6 5 4 taps are inside; no row padding."""
    acc = orc.conv_acc_i8(np.ones((1, 2, 9, 1), np.int8), np.ones((1, 1, 7, 1), np.int8), None, 1, 0, pad_w=3)[0, :, :, 0]
    assert acc.shape == (2, 9) and acc[0].tolist() == [4, 5, 6, 7, 7, 7, 6, 5, 4] and acc[1].tolist() == acc[0].tolist()


def test_avgpool_definition_and_closed_forms(orc):
    """k x k average with padding counted as zero and the divisor fixed at k*k, rounded half up."""
    from fractions import Fraction
    import math
    x = rand_i8(2, 6, 7, 3)
    y = orc.avgpool_i8(x, 3, 1, 1)
    assert y.shape == x.shape
    xp = np.pad(x.astype(np.int64), ((0, 0), (1, 1), (1, 1), (0, 0)))
    for (b, i, j, c) in [(0, 0, 0, 0), (1, 5, 6, 2), (0, 2, 3, 1), (1, 0, 4, 0), (0, 5, 0, 2)]:
        exact = Fraction(int(xp[b, i:i + 3, j:j + 3, c].sum()), 9)
        assert y[b, i, j, c] == math.floor(exact + Fraction(1, 2))
    ref = F.avg_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), 3, 1, 1, count_include_pad=True).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(y.astype(np.float64), np.floor(ref + 0.5))       # sums of 9 int8 over 9: no ties hidden by rounding in double
    const = np.full((1, 5, 5, 2), 90, np.int8)
    yc = orc.avgpool_i8(const, 3, 1, 1)
    assert np.all(yc[0, 1:-1, 1:-1] == 90) and yc[0, 0, 0, 0] == 40 and yc[0, 0, 2, 0] == 60     # 4/9 and 6/9 of 90 at corner and edge
    neg = np.full((1, 3, 3, 1), -128, np.int8)
    assert orc.avgpool_i8(neg, 3, 1, 1)[0, 1, 1, 0] == -128 and orc.avgpool_i8(neg, 3, 1, 1)[0, 0, 0, 0] == -57   # -512/9 = -56.9 -> -57
    half = np.array([1, 0, 0, 0, 0, 0, 0, 0, 0], np.int8).reshape(1, 3, 3, 1) * 0 + 0
    half[0, 1, 1, 0] = -5                                                   # -5/9 = -0.56 -> -1 ; 4/9 -> 0 ; 5/9 = 0.56 -> 1
    assert orc.avgpool_i8(half, 3, 1, 1)[0, 1, 1, 0] == -1
    half[0, 1, 1, 0] = 4
    assert orc.avgpool_i8(half, 3, 1, 1)[0, 1, 1, 0] == 0
    half[0, 1, 1, 0] = 5
    assert orc.avgpool_i8(half, 3, 1, 1)[0, 1, 1, 0] == 1
    # bf16: exact for small integers
    from workloads.blob import f32_to_bf16_bits, bf16_bits_to_f32
    xb = f32_to_bf16_bits(np.arange(25, dtype=np.float32).reshape(1, 5, 5, 1) * 9)
    yb = bf16_bits_to_f32(orc.avgpool_bf16(xb, 3, 1, 1))
    assert yb[0, 2, 2, 0] == 12 * 9 and yb[0, 0, 0, 0] == (0 + 9 + 45 + 54) / 9


def test_conv_1x1_is_a_gemm(orc):
    x, wt = rand_i8(2, 6, 5, 24), rand_i8(10, 1, 1, 24)
    acc = orc.conv_acc_i8(x, wt, None, 1, 0)
    gemm = x.reshape(-1, 24).astype(np.int64) @ wt.reshape(10, 24).astype(np.int64).T
    assert np.array_equal(acc.reshape(-1, 10), gemm)


def test_conv_identity_kernel_reproduces_input(orc):
    c = 6
    x = rand_i8(2, 7, 9, c)
    wt = np.zeros((c, 3, 3, c), np.int8)
    wt[np.arange(c), 1, 1, np.arange(c)] = 1
    assert np.array_equal(orc.conv_acc_i8(x, wt, None, 1, 1), x.astype(np.int32))
    assert np.array_equal(orc.requant_i8(orc.conv_acc_i8(x, wt, None, 1, 1), None, 0, 0, -128, 127), x)


def test_conv_all_ones_counts_in_range_taps(orc):
    acc = orc.conv_acc_i8(np.ones((1, 5, 6, 1), np.int8), np.ones((1, 3, 3, 1), np.int8), None, 1, 1)[0, :, :, 0]
    assert acc[0, 0] == 4 and acc[0, -1] == 4 and acc[-1, 0] == 4 and acc[-1, -1] == 4
    assert np.all(acc[0, 1:-1] == 6) and np.all(acc[1:-1, 0] == 6)
    assert np.all(acc[1:-1, 1:-1] == 9)


def test_conv_hand_example(orc):
    # 3x3 single-channel input, 2x2 kernel, no padding, worked by hand:
    #   [1 2 3; 4 5 6; 7 8 9] (*) [1 0; -1 2]  ->  [1-4+10, 2-5+12; 4-7+16, 5-8+18] = [7 9; 13 15]
    x = np.arange(1, 10, dtype=np.int8).reshape(1, 3, 3, 1)
    wt = np.array([1, 0, -1, 2], np.int8).reshape(1, 2, 2, 1)
    assert orc.conv_acc_i8(x, wt, np.array([100], np.int32), 1, 0)[0, :, :, 0].tolist() == [[107, 109], [113, 115]]


def test_conv_overflow_is_reported(orc):
    x = np.full((1, 1, 1, 8), 127, np.int8)
    wt = np.full((1, 1, 1, 8), 127, np.int8)
    with pytest.raises(orc.OracleError) as e:
        orc.conv_acc_i8(x, wt, np.array([2**31 - 1], np.int32), 1, 0)
    assert e.value.code == orc.ERR_OVERFLOW


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_equals_grouped_and_block_diagonal_conv(orc, stride):
    c = 5
    x, wt = rand_i8(2, 9, 8, c), rand_i8(c, 3, 3)
    bias = RNG.integers(-300, 300, size=c).astype(np.int32)
    acc = orc.dwconv_acc_i8(x, wt, bias, stride, 1)
    dense = np.zeros((c, 3, 3, c), np.int8)
    dense[np.arange(c), :, :, np.arange(c)] = wt
    assert np.array_equal(acc, orc.conv_acc_i8(x, dense, bias, stride, 1))
    ref = torch_conv(x, wt[..., None], bias, stride, 1, groups=c)
    assert np.array_equal(acc.astype(np.float64), ref)


def test_requant_exhaustive_against_rationals(orc):
    acc = np.arange(-4096, 4097, dtype=np.int32)
    for s in range(0, 9):
        y = orc.requant_i8(acc, None, s, 0, -128, 127)
        for a, q in zip(acc.tolist()[::7], y.tolist()[::7]):
            exact = (Fraction(a, 2**s) + Fraction(1, 2)).__floor__()   # round half up (towards +inf)
            assert q == max(-128, min(127, exact)), (a, s)
    assert orc.requant_i8(np.array([10**6, -10**6], np.int32), None, 3, 0, 0, 127).tolist() == [127, 0]
    assert orc.requant_i8(np.array([10**6, -10**6], np.int32), None, 3, 0, -128, 96).tolist() == [96, -128]
    # ties: -3/2 -> -1, 3/2 -> 2, -1/2 -> 0
    assert orc.requant_i8(np.array([-3, 3, -1], np.int32), None, 1, 0, -128, 127).tolist() == [-1, 2, 0]


def test_residual_identity_block(orc):
    x = rand_i8(1, 4, 4, 8)
    res = rand_i8(1, 4, 4, 8)
    acc = orc.conv_acc_i8(x, np.zeros((8, 3, 3, 8), np.int8), None, 1, 1)
    for s in (0, 3, 9):
        assert np.array_equal(orc.requant_i8(acc, res, s, s, -128, 127), res)
    # residual enters with weight 2^(res_shift - shift)
    y = orc.requant_i8(np.full(4, 64, np.int32), np.array([10, -10, 3, -3], np.int8), 6, 5, -128, 127)
    assert y.tolist() == [6, -4, 3, 0]          # 1 + r/2 rounded half up: 6, -4, 2.5->3, -0.5->0


def test_maxpool_matches_library(orc):
    x = rand_i8(2, 9, 11, 4)
    y = orc.maxpool_i8(x, 3, 2, 1)
    ref = F.max_pool2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(y.astype(np.float64), ref)
    allmin = np.full((1, 4, 4, 1), -128, np.int8)
    assert np.all(orc.maxpool_i8(allmin, 3, 2, 1) == -128)   # padding never wins


def test_gap_and_fc_closed_forms(orc):
    x = np.full((2, 7, 5, 3), 0, np.int8)
    x[0] = 9
    x[1, :, :, 1] = -4
    sums, g = orc.gap_i8(x, 5)
    assert sums.tolist() == [[315, 315, 315], [0, -140, 0]]
    assert g.tolist() == [[10, 10, 10], [0, -4, 0]]            # 315/32 = 9.84 -> 10 ; -140/32 = -4.375 -> -4
    xr = rand_i8(3, 6, 6, 10)
    sums, g = orc.gap_i8(xr, 6)
    assert np.array_equal(sums, xr.astype(np.int64).sum(axis=(1, 2)))
    onehot = np.eye(10, dtype=np.int8)[[3, 7, 0]]
    a = orc.fc_i8(g, onehot, np.array([5, -5, 0], np.int32))
    assert np.array_equal(a, g[:, [3, 7, 0]].astype(np.int32) + np.array([5, -5, 0]))
    w = rand_i8(12, 10)
    assert np.array_equal(orc.fc_i8(g, w, None), g.astype(np.int64) @ w.astype(np.int64).T)
    assert orc.gap_i8(np.full((1, 2, 2, 1), 127, np.int8), 0)[1].tolist() == [[127]]   # clamp after shift 0: 508 -> 127


def test_exp2_table_against_high_precision(orc):
    getcontext().prec = 60
    t = orc.exp2_table()
    ln2 = Decimal(2).ln()
    for i in range(256):
        exact = (Decimal(2) ** 30) * (-(Decimal(i) / 256) * ln2).exp()
        assert int(t[i]) == int(exact.to_integral_value(rounding="ROUND_HALF_EVEN")), i
    assert int(t[0]) == 1 << 30 and int(t[128]) == 759250125        # 2^29.5 rounded


def test_integer_softmax_closed_forms(orc):
    f = 10
    one = 1 << 30
    lab, s = orc.softmax_top1_i8(np.full((1, 10), 123, np.int32), f)
    assert lab[0] == 0 and s[0] == 10 * one                                   # all equal: conf = 1/K exactly
    a = np.full((1, 1000), -40 << f, np.int32)
    a[0, 417] = 0
    lab, s = orc.softmax_top1_i8(a, f)
    assert lab[0] == 417 and s[0] == one                                      # one far ahead: conf = 1
    a[0, 900] = 0
    lab, s = orc.softmax_top1_i8(a, f)
    assert lab[0] == 417 and s[0] == 2 * one                                  # two equal maxima: conf = 1/2, lowest index wins
    a = np.array([[0, -(1 << f), -(2 << f), -(30 << f), -(31 << f)]], np.int32)
    assert orc.softmax_top1_i8(a, f)[1][0] == one + one // 2 + one // 4 + 1 + 0   # whole powers of two, cut-off at 31
    # fraction bits: d = 2^(f-1) is half an octave -> table entry 128
    assert orc.softmax_top1_i8(np.array([[0, -(1 << (f - 1))]], np.int32), f)[1][0] == one + 759250125
    # f < 8: the fraction is left-aligned into the 8-bit table index
    assert orc.softmax_top1_i8(np.array([[0, -1]], np.int32), 1)[1][0] == one + 759250125


@pytest.mark.parametrize("f", [3, 8, 12])
def test_integer_softmax_close_to_real_softmax(orc, f):
    a = RNG.integers(-(6 << f), 6 << f, size=(50, 100)).astype(np.int32)
    lab, s = orc.softmax_top1_i8(a, f)
    z = a.astype(np.float64) * 2.0 ** -f
    p = np.exp2(z - z.max(axis=1, keepdims=True))
    conf_ref = 1.0 / p.sum(axis=1)
    conf = 2.0 ** 30 / s
    assert np.array_equal(lab, z.argmax(axis=1))
    rel = np.abs(conf - conf_ref) / conf_ref
    assert np.all(rel <= 2 ** (1 / 256) - 1 + 100 * 2.0 ** -30)             # table step + truncation bound
    assert np.all(conf <= conf_ref * (1 + 1e-9)) or np.all(rel < 3e-3)


def test_score_threshold_edges(orc):
    assert orc.score_threshold(0.0) == 2**63 - 1 and orc.score_threshold(-1.0) == 2**63 - 1
    assert orc.score_threshold(1.5) == 0
    assert orc.score_threshold(1.0) == 1 << 30
    assert orc.score_threshold(0.5) == 1 << 31
    assert orc.score_threshold(0.8) == int(np.floor(2.0**30 / float(np.float32(0.8))))


# ---- bf16 primitives -----------------------------------------------------------------
def to_bf16(a):
    from workloads import f32_to_bf16_bits
    return f32_to_bf16_bits(np.asarray(a, np.float32))


def from_bf16(b):
    from workloads import bf16_bits_to_f32
    return bf16_bits_to_f32(b)


def test_bf16_rounding(orc):
    lib = orc.lib()
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to the even mantissa (1.0)
    assert lib.orc_f32_to_bf16(1.0 + 2.0**-8) == 0x3F80
    assert lib.orc_f32_to_bf16(1.0 + 2.0**-7 + 2.0**-8) == 0x3F82
    assert lib.orc_f32_to_bf16(1.0 + 2.0**-8 + 2.0**-20) == 0x3F81
    vals = RNG.normal(size=1000).astype(np.float32)
    ours = np.array([lib.orc_f32_to_bf16(float(v)) for v in vals], np.uint16)
    assert np.array_equal(ours, torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(ours, to_bf16(vals))


def test_bf16_conv_small_integers_exact_and_library(orc):
    x = RNG.integers(-8, 9, size=(2, 6, 7, 4)).astype(np.float32)
    w = RNG.integers(-4, 5, size=(5, 3, 3, 4)).astype(np.float32)
    y = from_bf16(orc.conv_bf16(to_bf16(x), to_bf16(w), None, 1, 1))
    ref = torch_conv(x, w, None, 1, 1)
    assert np.array_equal(y.astype(np.float64), from_bf16(to_bf16(ref.astype(np.float32))).astype(np.float64))
    # general values: double accumulation, one rounding to float, then bf16
    xg, wg = RNG.normal(size=(1, 5, 5, 8)).astype(np.float32), RNG.normal(size=(6, 3, 3, 8)).astype(np.float32) * 0.2
    xb, wb = to_bf16(xg), to_bf16(wg)
    bias = RNG.normal(size=6).astype(np.float32)
    res = to_bf16(RNG.normal(size=(1, 3, 3, 6)).astype(np.float32))
    y = orc.conv_bf16(xb, wb, bias, 2, 1, res, 0.0, 1.5)
    accd = torch_conv(from_bf16(xb), from_bf16(wb), None, 2, 1)
    v = accd.astype(np.float32) + bias
    v = v + from_bf16(res)
    ref = to_bf16(np.clip(v, 0.0, 1.5))
    assert np.array_equal(y, ref)


def test_bf16_head_matches_double_softmax(orc):
    x = to_bf16(RNG.normal(size=(3, 4, 4, 16)).astype(np.float32))
    w = to_bf16(RNG.normal(size=(10, 16)).astype(np.float32))
    b = RNG.normal(size=10).astype(np.float32)
    logits, label, conf = orc.head_bf16(x, w, b, 1.7)
    g = from_bf16(x).astype(np.float64).mean(axis=(1, 2)).astype(np.float32)
    z = (1.7 * (g.astype(np.float64) @ from_bf16(w).astype(np.float64).T + b)).astype(np.float32)
    assert np.allclose(logits, z, rtol=1e-6, atol=1e-6)
    p = torch.softmax(torch.from_numpy(z.astype(np.float64)), dim=1).numpy()
    assert np.array_equal(label, p.argmax(axis=1))
    assert np.allclose(conf, p.max(axis=1), rtol=1e-6)


# ---- bf16 pooling and depthwise: library routines on bf16-exact values, closed forms, padding ----------
def _nchw(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64)).permute(0, 3, 1, 2)


def _nhwc(t):
    return t.permute(0, 2, 3, 1).numpy()


@pytest.mark.parametrize("k,stride,pad", [(3, 2, 1), (3, 1, 1), (2, 2, 0), (3, 2, 0), (5, 1, 2)])
def test_bf16_maxpool_matches_library_and_padding_never_wins(orc, k, stride, pad):
    """Max over the in-range taps only: the library's max-pool pads with -inf, which is the same statement.
    Values are small integers and halves, all exact in bf16, negative ones included so that a zero
    standing in for padding would win somewhere along the border."""
    x = (RNG.integers(-40, 41, size=(2, 9, 11, 5)) * 0.5).astype(np.float32)
    y = from_bf16(orc.maxpool_bf16(to_bf16(x), k, stride, pad))
    ref = _nhwc(F.max_pool2d(_nchw(x), k, stride, pad))
    assert y.shape == ref.shape and np.array_equal(y.astype(np.float64), ref)
    neg = np.full((1, 6, 6, 2), -3.0, np.float32)
    assert np.all(from_bf16(orc.maxpool_bf16(to_bf16(neg), k, stride, pad)) == -3.0)
    # a single peak is seen by exactly the windows that cover it (catches a transposed or shifted window)
    peak = np.full((1, 7, 8, 1), -1.0, np.float32)
    peak[0, 2, 5, 0] = 7.0
    yp = from_bf16(orc.maxpool_bf16(to_bf16(peak), k, stride, pad))[0, :, :, 0]
    for yo in range(yp.shape[0]):
        for xo in range(yp.shape[1]):
            covers = yo * stride - pad <= 2 < yo * stride - pad + k and xo * stride - pad <= 5 < xo * stride - pad + k
            assert yp[yo, xo] == (7.0 if covers else -1.0), (yo, xo)


def test_bf16_maxpool_returns_the_input_bits(orc):
    """The result is one of the inputs, bit for bit (-0.0 and denormals included), never a re-rounded float."""
    x = np.array([0x8000, 0x0001, 0xBF80, 0x8001], np.uint16).reshape(1, 2, 2, 1)       # -0.0, tiny, -1.0, -tiny
    assert int(orc.maxpool_bf16(x, 2, 2, 0)[0, 0, 0, 0]) == 0x0001
    x2 = np.array([0xBF80, 0xC000, 0xC040, 0xBFC0], np.uint16).reshape(1, 2, 2, 1)      # -1, -2, -3, -1.5
    assert int(orc.maxpool_bf16(x2, 2, 2, 0)[0, 0, 0, 0]) == 0xBF80


@pytest.mark.parametrize("stride", [1, 2])
def test_bf16_depthwise_matches_grouped_library_conv_and_dense_block_diagonal(orc, stride):
    c = 6
    x = RNG.integers(-8, 9, size=(2, 9, 8, c)).astype(np.float32)
    w = RNG.integers(-4, 5, size=(c, 3, 3)).astype(np.float32)
    bias = RNG.integers(-16, 17, size=c).astype(np.float32)
    y = from_bf16(orc.dwconv_bf16(to_bf16(x), to_bf16(w), bias, stride, 1))
    # sums stay below 2^8 * 9 * 4: exact in float, and exactly representable in bf16 only after rounding -> round the reference
    ref = torch_conv(x, w[..., None], bias, stride, 1, groups=c)
    assert y.shape == ref.shape
    assert np.array_equal(y.astype(np.float64), from_bf16(to_bf16(ref.astype(np.float32))).astype(np.float64))
    dense = np.zeros((c, 3, 3, c), np.float32)
    dense[np.arange(c), :, :, np.arange(c)] = w
    assert np.array_equal(to_bf16(y), orc.conv_bf16(to_bf16(x), to_bf16(dense), bias, stride, 1))
    # clamp (ReLU6-style) is applied after the bias
    yc = from_bf16(orc.dwconv_bf16(to_bf16(x), to_bf16(w), bias, stride, 1, 0.0, 6.0))
    assert np.array_equal(yc.astype(np.float64), np.clip(from_bf16(to_bf16(ref.astype(np.float32))), 0.0, 6.0).astype(np.float64))


def test_bf16_depthwise_tap_counts_and_hand_example(orc):
    ones = to_bf16(np.ones((1, 4, 5, 2), np.float32))
    y = from_bf16(orc.dwconv_bf16(ones, to_bf16(np.ones((2, 3, 3), np.float32)), None, 1, 1))[0, :, :, 0]
    assert y[0, 0] == 4 and y[0, 2] == 6 and y[1, 0] == 6 and y[1, 2] == 9 and y[3, 4] == 4
    # channel 1 of a 3x3 input with kernel [[0,0,0],[0,0,1],[0,2,0]] (no padding): x[1][2] + 2 x[2][1]
    x = np.zeros((1, 3, 3, 2), np.float32)
    x[0, :, :, 1] = np.arange(9).reshape(3, 3)
    w = np.zeros((2, 3, 3), np.float32)
    w[1, 1, 2], w[1, 2, 1] = 1.0, 2.0
    out = from_bf16(orc.dwconv_bf16(to_bf16(x), to_bf16(w), np.array([0.5, 0.25], np.float32), 1, 0))
    assert out.shape == (1, 1, 1, 2) and out[0, 0, 0].tolist() == [0.5, 5 + 2 * 7 + 0.25]


@pytest.mark.parametrize("k,stride,pad", [(3, 1, 1), (3, 2, 1), (2, 2, 0), (5, 1, 2)])
def test_bf16_avgpool_matches_library_on_exact_values(orc, k, stride, pad):
    """Padding counts as zero and the divisor is k*k everywhere (the library's count_include_pad).  The inputs are
    multiples of k*k small enough that every window mean is an integer below 256: exact in bf16, no rounding involved."""
    x = (RNG.integers(-5, 6, size=(2, 8, 9, 3)) * (k * k)).astype(np.float32)
    y = from_bf16(orc.avgpool_bf16(to_bf16(x), k, stride, pad))
    ref = _nhwc(F.avg_pool2d(_nchw(x), k, stride, pad, count_include_pad=True))
    assert y.shape == ref.shape and np.array_equal(y.astype(np.float64), ref)


def test_bf16_avgpool_rounds_once(orc):
    """General values: the window sum in double divided by k*k, one rounding to float and one to bf16."""
    x = to_bf16(RNG.normal(size=(1, 6, 7, 4)).astype(np.float32))
    y = orc.avgpool_bf16(x, 3, 1, 1)
    ref = _nhwc(F.avg_pool2d(_nchw(from_bf16(x)), 3, 1, 1, count_include_pad=True))       # float64
    assert np.array_equal(y, to_bf16(ref.astype(np.float32)))
    corner = to_bf16(np.full((1, 3, 3, 1), 9.0, np.float32))
    yc = from_bf16(orc.avgpool_bf16(corner, 3, 1, 1))[0, :, :, 0]
    assert yc[0, 0] == 4.0 and yc[0, 1] == 6.0 and yc[1, 1] == 9.0                        # 4, 6 and 9 taps of 9 over the fixed divisor 9
