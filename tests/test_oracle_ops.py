"""Pins of the operator oracle against things other than itself.

Each check is chosen so that a plausible slip in ``oracle/tt_oracle.c`` (a
dropped term, a flipped filter, swapped strides or pads, a transposed operand,
bias or residual applied after the activation) fails at least one of them.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import ops


def rng(seed):
    return np.random.default_rng(seed)


# ---- brute force with a different loop order and Python floats (double) -------------------------
def conv_brute(x, w, bias, res, stride, pad, act):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    xp = np.zeros((n, c, h + 2 * pad[0], wd + 2 * pad[1]), dtype=np.float64)
    xp[:, :, pad[0]:pad[0] + h, pad[1]:pad[1] + wd] = x
    ho = (h + 2 * pad[0] - r) // stride[0] + 1
    wo = (wd + 2 * pad[1] - s) // stride[1] + 1
    y = np.zeros((n, k, ho, wo), dtype=np.float64)
    # taps outermost: scatter each (r, s, c) contribution into the whole output
    for ri, si, ci in itertools.product(range(r), range(s), range(c)):
        for ni, ki, p, q in itertools.product(range(n), range(k), range(ho), range(wo)):
            y[ni, ki, p, q] += xp[ni, ci, p * stride[0] + ri, q * stride[1] + si] * float(w[ki, ci, ri, si])
    if bias is not None:
        y += bias.astype(np.float64)[None, :, None, None]
    if res is not None:
        y += res
    if act == ops.ACT_RELU:
        y = np.maximum(y, 0)
    elif act == ops.ACT_RELU6:
        y = np.clip(y, 0, 6)
    return y


@pytest.mark.parametrize("stride,pad,rs", [((1, 1), (1, 1), (3, 3)), ((2, 2), (1, 1), (3, 3)),
                                           ((2, 1), (0, 2), (2, 3)), ((1, 2), (3, 0), (7, 1)),
                                           ((2, 2), (0, 0), (1, 1))])
def test_conv_brute_force_tiny(stride, pad, rs):
    g = rng(1)
    x = g.uniform(-1, 1, (2, 3, 6, 5)).astype(np.float32)
    w = g.standard_normal((4, 3) + rs).astype(np.float32)
    b = g.uniform(-0.5, 0.5, 4).astype(np.float32)
    ref = conv_brute(x, w, b, None, stride, pad, ops.ACT_RELU)
    got = ops.conv2d(x, w, b, None, stride, pad, ops.ACT_RELU)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)
    res = g.uniform(-1, 1, ref.shape).astype(np.float32)
    ref = conv_brute(x, w, b, res, stride, pad, ops.ACT_RELU)
    np.testing.assert_allclose(ops.conv2d(x, w, b, res, stride, pad, ops.ACT_RELU), ref, rtol=1e-6, atol=1e-6)
    ref = conv_brute(x, w, b, None, stride, pad, ops.ACT_NONE)
    np.testing.assert_allclose(ops.conv2d(x, w, b, None, stride, pad, ops.ACT_NONE), ref, rtol=1e-6, atol=1e-6)


def test_conv_output_extent_closed_form():
    # ResNet stem: 224 -> 112 with 7x7/s2/p3; 3x3/s2/p1 halves 56 -> 28; 1x1/s2 halves 14 -> 7
    assert ops.conv_out_extent(224, 7, 2, 3) == 112
    assert ops.conv_out_extent(56, 3, 2, 1) == 28
    assert ops.conv_out_extent(14, 1, 2, 0) == 7
    assert ops.conv_out_extent(7, 3, 1, 1) == 7


def test_conv_1x1_is_matmul():
    g = rng(2)
    x = g.standard_normal((2, 5, 4, 3)).astype(np.float32)
    w = g.standard_normal((6, 5, 1, 1)).astype(np.float32)
    got = ops.conv2d(x, w)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)


def test_conv_delta_filter_is_identity_plus_bias():
    g = rng(3)
    c = 4
    x = g.uniform(-1, 1, (1, c, 7, 6)).astype(np.float32)
    b = g.uniform(-0.1, 0.1, c).astype(np.float32)
    w = np.zeros((c, c, 3, 3), dtype=np.float32)
    for i in range(c):
        w[i, i, 1, 1] = 1.0
    got = ops.conv2d(x, w, b, None, (1, 1), (1, 1), ops.ACT_RELU)
    np.testing.assert_array_equal(got, np.maximum(x + b[None, :, None, None], 0).astype(np.float32))


def test_conv_off_centre_delta_is_a_shift_not_a_flip():
    # cross-correlation: a tap at (r=0, s=2) reads the input up one row and right one column
    x = np.arange(2 * 5 * 5, dtype=np.float32).reshape(1, 2, 5, 5)
    w = np.zeros((2, 2, 3, 3), dtype=np.float32)
    w[0, 0, 0, 2] = 1.0
    w[1, 1, 2, 0] = 1.0
    got = ops.conv2d(x, w, None, None, (1, 1), (1, 1))
    ref = np.zeros_like(x)
    ref[0, 0, 1:, :-1] = x[0, 0, :-1, 1:]
    ref[0, 1, :-1, 1:] = x[0, 1, 1:, :-1]
    np.testing.assert_array_equal(got, ref)


def test_conv_zero_filter_gives_activation_of_bias():
    x = rng(4).uniform(-1, 1, (1, 3, 5, 5)).astype(np.float32)
    b = np.array([-0.5, 0.25, 7.0], dtype=np.float32)
    w = np.zeros((3, 3, 3, 3), dtype=np.float32)
    got = ops.conv2d(x, w, b, None, (1, 1), (1, 1), ops.ACT_RELU)
    for k, v in enumerate([0.0, 0.25, 7.0]):
        assert np.all(got[:, k] == np.float32(v))
    got6 = ops.conv2d(x, w, b, None, (1, 1), (1, 1), ops.ACT_RELU6)
    assert np.all(got6[:, 2] == 6.0)


def test_conv_linearity_and_relu_nonnegative():
    g = rng(5)
    x = g.uniform(-1, 1, (1, 4, 8, 8)).astype(np.float32)
    w1 = g.standard_normal((5, 4, 3, 3)).astype(np.float32)
    w2 = g.standard_normal((5, 4, 3, 3)).astype(np.float32)
    y1 = ops.conv2d(x, w1, None, None, (2, 2), (1, 1))
    y2 = ops.conv2d(x, w2, None, None, (2, 2), (1, 1))
    y12 = ops.conv2d(x, (w1.astype(np.float64) + 2 * w2).astype(np.float32), None, None, (2, 2), (1, 1))
    np.testing.assert_allclose(y12, y1 + 2 * y2, rtol=1e-5, atol=1e-5)
    assert ops.conv2d(x, w1, None, None, (2, 2), (1, 1), ops.ACT_RELU).min() >= 0.0


def test_conv_shift_equivariance_in_the_interior():
    g = rng(6)
    x = g.uniform(-1, 1, (1, 2, 10, 10)).astype(np.float32)
    w = g.standard_normal((3, 2, 3, 3)).astype(np.float32)
    y = ops.conv2d(x, w, None, None, (1, 1), (1, 1))
    xs = np.roll(x, (1, 2), axis=(2, 3))
    ys = ops.conv2d(xs, w, None, None, (1, 1), (1, 1))
    np.testing.assert_allclose(ys[:, :, 3:-1, 4:-1], y[:, :, 2:-2, 2:-3], rtol=1e-6, atol=1e-6)


def test_residual_and_bias_are_added_before_the_activation():
    x = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    b = np.array([1.0], dtype=np.float32)
    res = np.full((1, 1, 3, 3), -3.0, dtype=np.float32)
    got = ops.conv2d(x, w, b, res, (1, 1), (1, 1), ops.ACT_RELU)
    assert np.all(got == 0.0)  # relu(1 - 3) = 0, not relu(1) - 3


# ---- dense / batch matmul ------------------------------------------------------------------------
def test_dense_against_library_matmul_and_identity():
    g = rng(7)
    x = g.standard_normal((5, 7)).astype(np.float32)
    w = g.standard_normal((3, 7)).astype(np.float32)
    b = g.uniform(-1, 1, 3).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    np.testing.assert_allclose(ops.dense(x, w, b), ref, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(ops.dense(x, w, b, ops.ACT_RELU), np.maximum(ref, 0), rtol=1e-6, atol=1e-6)
    np.testing.assert_array_equal(ops.dense(x, np.eye(7, dtype=np.float32)), x)


def test_gelu_exact_form_values():
    x = np.array([[-3.0, -1.0, 0.0, 0.5, 1.0, 4.0]], dtype=np.float32)
    got = ops.dense(x, np.eye(6, dtype=np.float32), None, ops.ACT_GELU)[0]
    ref = [0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x[0]]
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-7)
    # known values of x * Phi(x): Phi(1) = 0.8413447460685429
    assert abs(got[4] - 0.8413447460685429) < 1e-6 and got[2] == 0.0


def test_batch_matmul_layouts_and_transpose_rule():
    g = rng(8)
    a = g.standard_normal((3, 4, 6)).astype(np.float32)
    b = g.standard_normal((3, 6, 5)).astype(np.float32)
    ref = np.einsum("bmk,bkn->bmn", a.astype(np.float64), b.astype(np.float64))
    c0 = ops.batch_matmul(a, b, trans_b=False)
    np.testing.assert_allclose(c0, ref, rtol=1e-6, atol=1e-6)
    c1 = ops.batch_matmul(a, np.ascontiguousarray(b.transpose(0, 2, 1)), trans_b=True)
    np.testing.assert_array_equal(c0, c1)
    # (A B)^T = B^T A^T
    ct = ops.batch_matmul(np.ascontiguousarray(b.transpose(0, 2, 1)), np.ascontiguousarray(a.transpose(0, 2, 1)))
    np.testing.assert_allclose(ct, c0.transpose(0, 2, 1), rtol=1e-6, atol=1e-6)


def test_dense_is_batch_matmul_with_one_batch():
    g = rng(9)
    x = g.standard_normal((6, 9)).astype(np.float32)
    w = g.standard_normal((4, 9)).astype(np.float32)
    np.testing.assert_array_equal(ops.dense(x, w), ops.batch_matmul(x[None], w[None], trans_b=True)[0])


# ---- depthwise -----------------------------------------------------------------------------------
@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_equals_dense_conv_with_block_diagonal_weights(stride):
    g = rng(10)
    c = 5
    x = g.uniform(-3, 3, (2, c, 9, 8)).astype(np.float32)
    w = g.standard_normal((c, 1, 3, 3)).astype(np.float32)
    b = g.uniform(-1, 1, c).astype(np.float32)
    full = np.zeros((c, c, 3, 3), dtype=np.float32)
    for i in range(c):
        full[i, i] = w[i, 0]
    ref = ops.conv2d(x, full, b, None, (stride, stride), (1, 1), ops.ACT_RELU6)
    got = ops.dwconv(x, w, b, (stride, stride), (1, 1), ops.ACT_RELU6)
    np.testing.assert_array_equal(got, ref)
    assert got.min() >= 0.0 and got.max() <= 6.0
    ref2 = conv_brute(x, full, b, None, (stride, stride), (1, 1), ops.ACT_RELU6)
    np.testing.assert_allclose(got, ref2, rtol=1e-6, atol=1e-6)


def test_depthwise_delta_is_clamped_identity():
    x = np.linspace(-8, 8, 2 * 3 * 4 * 4, dtype=np.float32).reshape(2, 3, 4, 4)
    w = np.zeros((3, 1, 3, 3), dtype=np.float32)
    w[:, 0, 1, 1] = 1.0
    b = np.array([0.5, 0.0, -0.5], dtype=np.float32)
    got = ops.dwconv(x, w, b)
    np.testing.assert_array_equal(got, np.clip(x + b[None, :, None, None], 0, 6).astype(np.float32))


# ---- accumulators --------------------------------------------------------------------------------
def test_float_accumulator_stays_within_the_summation_error_bound():
    g = rng(11)
    k = 4608  # the longest reduction of the ResNet-shaped kernels (512 * 3 * 3)
    x = g.uniform(-1, 1, (4, k)).astype(np.float32)
    w = (g.standard_normal((8, k)) / np.sqrt(k)).astype(np.float32)
    y64 = ops.dense(x, w, acc64=True)
    y32 = ops.dense(x, w, acc64=False)
    absdot = np.abs(x.astype(np.float64)) @ np.abs(w.astype(np.float64)).T
    # recursive summation: |err| <= (K - 1) u sum|x_i w_i| + one rounding of each product; u = 2^-24
    assert np.all(np.abs(y32.astype(np.float64) - y64) <= (k + 1) * 2.0 ** -24 * absdot + 1e-12)
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.max(np.abs(y64 - exact)) <= 2.0 ** -23 * np.max(np.abs(exact)) + 1e-12


# ---- bf16 ----------------------------------------------------------------------------------------
def test_bf16_round_trip_over_every_code():
    for h in range(0, 1 << 16):
        f = ops.bf16_bits_to_f32(h)
        if math.isnan(f):
            continue
        assert ops.f32_to_bf16_bits(f) == h


def test_bf16_ties_go_to_even_and_carry():
    def f32(bits):
        return float(np.array([bits], dtype=np.uint32).view(np.float32)[0])
    assert ops.f32_to_bf16_bits(f32(0x3F808000)) == 0x3F80          # tie, even stays
    assert ops.f32_to_bf16_bits(f32(0x3F818000)) == 0x3F82          # tie, odd rounds up
    assert ops.f32_to_bf16_bits(f32(0x3F808001)) == 0x3F81          # just above the tie
    assert ops.f32_to_bf16_bits(f32(0x3F807FFF)) == 0x3F80          # just below
    assert ops.f32_to_bf16_bits(f32(0x3FFFFFFF)) == 0x4000          # mantissa carry into the exponent
    assert ops.f32_to_bf16_bits(f32(0x7F7FFFFF)) == 0x7F80          # largest float rounds to infinity
    assert ops.f32_to_bf16_bits(-0.0) == 0x8000
    assert ops.f32_to_bf16_bits(1.0 + 2.0 ** -8) == 0x3F80          # 1 + half ulp(bf16) ties to even
    assert ops.f32_to_bf16_bits(1.0 + 3 * 2.0 ** -8) == 0x3F82


def test_bf16_rounding_matches_library_conversion():
    import torch
    a = rng(12).standard_normal(200000).astype(np.float32) * 10.0
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(ops.round_to_bf16(a), ref)


def test_conv_points_agree_with_the_full_tensor():
    g = rng(13)
    x = g.uniform(-1, 1, (2, 5, 9, 8)).astype(np.float32)
    w = g.standard_normal((6, 5, 3, 3)).astype(np.float32)
    b = g.uniform(-1, 1, 6).astype(np.float32)
    full = ops.conv2d(x, w, b, None, (2, 1), (1, 1), ops.ACT_RELU)
    res = g.uniform(-1, 1, full.shape).astype(np.float32)
    full = ops.conv2d(x, w, b, res, (2, 1), (1, 1), ops.ACT_RELU)
    coords = np.array(list(itertools.product(range(2), range(6), range(full.shape[2]), range(full.shape[3]))), dtype=np.int32)
    pts = ops.conv2d_points(x, w, coords, b, res, (2, 1), (1, 1), ops.ACT_RELU)
    np.testing.assert_array_equal(pts, full.reshape(-1))
    with pytest.raises(ValueError):
        ops.conv2d_points(x, w, np.array([[0, 0, 99, 0]]), b)
