"""Pins for the oracle's neighbours of the convolution (no GPU needed): the two
fused epilogues (bias + ReLU behind the forward pass, ReLU mask on backward-data)
and training-mode batch normalisation with its vector-Jacobian product.

The paper names these operators (Section 4.1's model code; Section 6.1's
ResNet-50 trace) but prints no numbers for them, so they are pinned to closed
forms, hand-computed values, independent numpy constructions, invariants and
finite differences.  Each test is aimed at one plausible mistake (ReLU before
the bias, bias indexed by the wrong axis, mask taken from the wrong tensor,
variance without the mean removed, eps outside the root, unbiased variance,
statistics over the wrong axes, a dropped term of dx, ...).
"""
import numpy as np
import pytest

from oracle import convref as ref
from test_oracle_pins import im2col_conv

RNG = np.random.default_rng(20240911)


def rnd(*shape):
    return RNG.standard_normal(shape)


# ------------------------------------------------------------------ forward + bias + ReLU
def test_bias_relu_with_zero_bias_and_nonnegative_operands_is_the_plain_forward():
    x, w = np.abs(rnd(2, 4, 6, 5)), np.abs(rnd(6, 2, 3, 3))
    got = ref.conv2d_fwd_bias_relu(x, w, np.zeros(6), 1, 1, 2)
    assert np.array_equal(got, ref.conv2d_fwd(x, w, 1, 1, 2))


def test_bias_relu_all_ones_closed_form():
    # 3x3, padding 1, C channels of ones: 9C inside, 6C on edges, 4C in corners; then + bias[k], clamped at 0.
    C = 4
    x, w = np.ones((1, C, 5, 6)), np.ones((3, C, 3, 3))
    bias = np.array([0.5, -6.0 * C - 0.5, -100.0])
    y = ref.conv2d_fwd_bias_relu(x, w, bias, 1, 1)
    base = np.full((5, 6), 9.0 * C)
    base[0, :] = base[-1, :] = base[:, 0] = base[:, -1] = 6.0 * C
    base[0, 0] = base[0, -1] = base[-1, 0] = base[-1, -1] = 4.0 * C
    assert np.array_equal(y[0, 0], base + 0.5)
    exp1 = np.zeros((5, 6))
    exp1[1:-1, 1:-1] = 3.0 * C - 0.5          # only the interior stays positive
    assert np.array_equal(y[0, 1], exp1)
    assert np.array_equal(y[0, 2], np.zeros((5, 6)))


def test_bias_relu_everything_negative_gives_exact_zero():
    x, w = np.abs(rnd(2, 3, 5, 5)) + 0.1, -np.abs(rnd(4, 3, 3, 3)) - 0.1
    y = ref.conv2d_fwd_bias_relu(x, w, -np.abs(rnd(4)), 1, 0)
    assert np.array_equal(y, np.zeros_like(y))


def test_relu_comes_after_the_bias():
    # one pixel, one channel, 1x1 filter: conv value = x*w
    one = lambda v: np.full((1, 1, 1, 1), float(v))
    assert ref.conv2d_fwd_bias_relu(one(-1), one(1), np.array([3.0]))[0, 0, 0, 0] == 2.0    # relu first would give 3
    assert ref.conv2d_fwd_bias_relu(one(1), one(1), np.array([-3.0]))[0, 0, 0, 0] == 0.0    # no relu: -2; relu first: -2


@pytest.mark.parametrize("N,C,H,W,K,R,S,st,pd,g", [
    (2, 3, 7, 6, 5, 3, 3, (1, 1), (1, 1), 1),
    (3, 4, 9, 8, 6, 3, 2, (2, 1), (0, 1), 2),      # N, K, P, Q all different: a bias indexed by another axis shows
    (1, 6, 8, 11, 6, 1, 3, (1, 3), (0, 2), 3),
])
def test_bias_relu_against_numpy_construction(N, C, H, W, K, R, S, st, pd, g):
    x, w, b = rnd(N, C, H, W), rnd(K, C // g, R, S), rnd(K)
    want = np.maximum(im2col_conv(x, w, st, pd, g) + b[None, :, None, None], 0.0)
    got = ref.conv2d_fwd_bias_relu(x, w, b, st, pd, g)
    assert got.shape == want.shape
    assert np.max(np.abs(got - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))
    assert np.array_equal(got == 0.0, want == 0.0)


def test_bias_relu_directional_derivative_is_the_masked_forward_of_the_direction():
    # F is piecewise linear in x: away from the kink, (F(x + h e) - F(x - h e)) / 2h = fwd(e, w) where the
    # pre-activation is positive and 0 where it is negative.
    x, w, b = rnd(2, 3, 6, 6), rnd(4, 3, 3, 3), rnd(4)
    pre = ref.conv2d_fwd(x, w, 1, 1) + b[None, :, None, None]
    h = 1e-3
    for flat in (0, 57, 101, 215):
        e = np.zeros(x.size)
        e[flat] = 1.0
        e = e.reshape(x.shape)
        lin = ref.conv2d_fwd(e, w, 1, 1)
        safe = np.abs(pre) > 2 * h * np.abs(lin) + 1e-9        # the step does not cross the kink
        diff = (ref.conv2d_fwd_bias_relu(x + h * e, w, b, 1, 1) - ref.conv2d_fwd_bias_relu(x - h * e, w, b, 1, 1)) / (2 * h)
        want = np.where(pre > 0, lin, 0.0)
        assert safe.mean() > 0.9
        assert np.max(np.abs(diff - want)[safe]) <= 1e-10


def test_bias_relu_widens_fp32_and_bf16_inputs_exactly():
    x32, w32 = rnd(1, 2, 5, 5).astype(np.float32), rnd(3, 2, 3, 3).astype(np.float32)
    b = rnd(3)
    assert np.array_equal(ref.conv2d_fwd_bias_relu(x32, w32, b, 1, 1),
                          ref.conv2d_fwd_bias_relu(x32.astype(np.float64), w32.astype(np.float64), b, 1, 1))
    xb = (x32.view(np.uint32) >> 16).astype(np.uint16)
    wb = (w32.view(np.uint32) >> 16).astype(np.uint16)
    widen = lambda u: (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.array_equal(ref.conv2d_fwd_bias_relu(xb, wb, b, 1, 1), ref.conv2d_fwd_bias_relu(widen(xb), widen(wb), b, 1, 1))


# ------------------------------------------------------------------ backward-data with ReLU mask
def test_relu_mask_all_positive_is_the_plain_backward_data():
    dy, w = rnd(2, 4, 3, 3), rnd(4, 3, 3, 3)
    act = np.abs(rnd(2, 3, 5, 5)) + 0.01
    assert np.array_equal(ref.conv2d_bwd_data_relu(dy, w, act, 2, 1), ref.conv2d_bwd_data(dy, w, act.shape, 2, 1))


def test_relu_mask_zeroes_exactly_where_the_activation_is_not_positive():
    dy, w = rnd(2, 6, 6, 7), rnd(6, 2, 3, 3)
    act = rnd(2, 4, 6, 7)
    act[0, 0, 0, :3] = [0.0, -0.0, 1e-300]       # zero and negative zero are masked, the smallest positive is not
    plain = ref.conv2d_bwd_data(dy, w, act.shape, 1, 1, 2)
    got = ref.conv2d_bwd_data_relu(dy, w, act, 1, 1, 2)
    assert np.array_equal(got[act > 0], plain[act > 0])
    assert np.array_equal(got[~(act > 0)], np.zeros(np.count_nonzero(~(act > 0))))
    assert got[0, 0, 0, 2] == plain[0, 0, 0, 2] and got[0, 0, 0, 0] == 0.0 and got[0, 0, 0, 1] == 0.0
    assert 0.3 < np.mean(act > 0) < 0.7          # the mask comes from act, not from dy or from the result


def test_relu_mask_bf16_sign_and_zero_patterns():
    dy = np.full((1, 1, 1, 4), 0x3F80, dtype=np.uint16)        # 1.0
    w = np.full((1, 1, 1, 1), 0x4000, dtype=np.uint16)         # 2.0
    act = np.array([0x0000, 0x8000, 0x0001, 0xBF80], dtype=np.uint16).reshape(1, 1, 1, 4)   # +0, -0, tiny > 0, -1
    got = ref.conv2d_bwd_data_relu(dy, w, act)
    assert np.array_equal(got.reshape(-1), [0.0, 0.0, 2.0, 0.0])


def test_relu_mask_is_the_gradient_of_the_composition_by_finite_differences():
    # L(z) = <conv2d_fwd(max(0, z), w), dy> is piecewise linear in z: central differences are exact away from 0.
    z, w = rnd(1, 2, 5, 5), rnd(3, 2, 3, 3)
    dy = rnd(1, 3, 3, 3)
    act = np.maximum(z, 0.0)
    got = ref.conv2d_bwd_data_relu(dy, w, act, 2, 1)
    L = lambda zz: float(np.sum(ref.conv2d_fwd(np.maximum(zz, 0.0), w, 2, 1) * dy))
    h = 1e-4
    checked = 0
    for flat in range(z.size):
        if abs(z.reshape(-1)[flat]) <= 2 * h:
            continue
        e = np.zeros(z.size)
        e[flat] = h
        e = e.reshape(z.shape)
        fd = (L(z + e) - L(z - e)) / (2 * h)
        assert abs(fd - got.reshape(-1)[flat]) <= 1e-9 * max(1.0, abs(fd))
        checked += 1
    assert checked >= 45


# ------------------------------------------------------------------ batch normalisation, forward
def test_bn_hand_example():
    # one channel with the values 1, 2, 3, 4 (N=2, H=1, W=2): mean 2.5, biased variance 1.25, eps = 0
    x = np.array([1.0, 2.0, 3.0, 4.0]).reshape(2, 1, 1, 2)
    y, mean, inv_std = ref.batchnorm2d_fwd(x, np.ones(1), np.zeros(1), 0.0)
    assert mean[0] == 2.5
    assert abs(inv_std[0] - 0.8944271909999159) <= 1e-15                      # 1 / sqrt(1.25) = 2 / sqrt(5)
    want = np.array([-1.3416407864998738, -0.4472135954999579, 0.4472135954999579, 1.3416407864998738])
    assert np.max(np.abs(y.reshape(-1) - want)) <= 1e-15
    # unbiased variance (5/3) would give 1/sqrt(5/3) = 0.7746


def test_bn_eps_sits_inside_the_root():
    x = np.array([1.0, -1.0, 1.0, -1.0]).reshape(4, 1, 1, 1)        # variance 1
    y, _, inv_std = ref.batchnorm2d_fwd(x, np.ones(1), np.zeros(1), 3.0)
    assert inv_std[0] == 0.5 and np.array_equal(y.reshape(-1), [0.5, -0.5, 0.5, -0.5])


def test_bn_constant_channel_gives_beta():
    x = np.empty((3, 2, 4, 5))
    x[:, 0], x[:, 1] = 7.25, -3.5
    y, mean, inv_std = ref.batchnorm2d_fwd(x, np.array([2.0, -1.5]), np.array([0.75, 4.0]), 1e-5)
    assert np.array_equal(mean, [7.25, -3.5])
    assert np.array_equal(y[:, 0], np.full((3, 4, 5), 0.75)) and np.array_equal(y[:, 1], np.full((3, 4, 5), 4.0))
    assert np.allclose(inv_std, 1.0 / np.sqrt(1e-5), rtol=1e-15)


def test_bn_statistics_run_over_batch_and_pixels_of_each_channel():
    # channel c is shifted by 10 c and scaled by c + 1: statistics over any other set of axes would mix them
    N, C, H, W = 5, 3, 4, 6
    base = rnd(N, C, H, W)
    x = base * (np.arange(C) + 1.0)[None, :, None, None] + 10.0 * np.arange(C)[None, :, None, None]
    eps = 1e-3
    y, mean, inv_std = ref.batchnorm2d_fwd(x, np.ones(C), np.zeros(C), eps)
    assert np.max(np.abs(mean - x.mean(axis=(0, 2, 3)))) <= 1e-13
    var = x.var(axis=(0, 2, 3))                                   # numpy's default is the biased variance
    assert np.max(np.abs(inv_std - 1.0 / np.sqrt(var + eps))) <= 1e-13
    assert np.max(np.abs(y.mean(axis=(0, 2, 3)))) <= 1e-13
    assert np.max(np.abs(y.var(axis=(0, 2, 3)) - var / (var + eps))) <= 1e-12
    want = (x - x.mean(axis=(0, 2, 3), keepdims=True)) / np.sqrt(x.var(axis=(0, 2, 3), keepdims=True) + eps)
    assert np.max(np.abs(y - want)) <= 1e-12


def test_bn_affine_part():
    x, g, b = rnd(3, 4, 5, 5), rnd(4), rnd(4)
    y0, m0, s0 = ref.batchnorm2d_fwd(x, np.ones(4), np.zeros(4), 1e-5)
    y1, m1, s1 = ref.batchnorm2d_fwd(x, g, b, 1e-5)
    assert np.array_equal(m0, m1) and np.array_equal(s0, s1)
    assert np.max(np.abs(y1 - (g[None, :, None, None] * y0 + b[None, :, None, None]))) <= 1e-14


def test_bn_is_invariant_to_shift_and_scale_of_the_input_without_eps():
    x = rnd(4, 2, 3, 3)
    y0, _, _ = ref.batchnorm2d_fwd(x, np.ones(2), np.zeros(2), 0.0)
    y1, _, _ = ref.batchnorm2d_fwd(-3.0 * x + 11.0, np.ones(2), np.zeros(2), 0.0)
    assert np.max(np.abs(y1 + y0)) <= 1e-12                       # a negative scale flips the sign


def test_bn_widens_fp32_and_bf16_exactly():
    x32 = rnd(2, 3, 4, 4).astype(np.float32)
    g, b = rnd(3), rnd(3)
    for a, wide in ((x32, x32.astype(np.float64)),
                    ((x32.view(np.uint32) >> 16).astype(np.uint16),
                     ((x32.view(np.uint32) >> 16) << 16).astype(np.uint32).view(np.float32).astype(np.float64))):
        for u, v in zip(ref.batchnorm2d_fwd(a, g, b, 1e-5), ref.batchnorm2d_fwd(wide, g, b, 1e-5)):
            assert np.array_equal(u, v)


# ------------------------------------------------------------------ batch normalisation, backward
def test_bn_backward_sums_and_orthogonality():
    N, C, H, W = 4, 3, 5, 6
    x, dy, g = rnd(N, C, H, W) * 2.0 + 1.0, rnd(N, C, H, W), rnd(C)
    eps = 1e-4
    dx, dgamma, dbeta = ref.batchnorm2d_bwd(x, dy, g, eps)
    xhat = (x - x.mean(axis=(0, 2, 3), keepdims=True)) / np.sqrt(x.var(axis=(0, 2, 3), keepdims=True) + eps)
    assert np.max(np.abs(dbeta - dy.sum(axis=(0, 2, 3)))) <= 1e-12
    assert np.max(np.abs(dgamma - (dy * xhat).sum(axis=(0, 2, 3)))) <= 1e-12
    # y does not change when x is shifted, so dx sums to zero per channel; and (for eps -> 0) not when it is scaled
    assert np.max(np.abs(dx.sum(axis=(0, 2, 3)))) <= 1e-12
    dx0, _, _ = ref.batchnorm2d_bwd(x, dy, g, 0.0)
    xc = x - x.mean(axis=(0, 2, 3), keepdims=True)
    assert np.max(np.abs((dx0 * xc).sum(axis=(0, 2, 3)))) <= 1e-11


def test_bn_backward_against_central_finite_differences():
    # L(x, gamma, beta) = <batchnorm(x; gamma, beta), dy>.  The map is smooth but not linear: with a step of 1e-5
    # the truncation error of a central difference is about 1e-10 and the rounding error about 1e-11; bound 1e-6.
    N, C, H, W = 3, 2, 3, 4
    x, dy, g, b = rnd(N, C, H, W) + 0.5, rnd(N, C, H, W), rnd(C) + 2.0, rnd(C)
    eps = 1e-2
    dx, dgamma, dbeta = ref.batchnorm2d_bwd(x, dy, g, eps)
    L = lambda xx, gg, bb: float(np.sum(ref.batchnorm2d_fwd(xx, gg, bb, eps)[0] * dy))
    h = 1e-5
    for flat in range(x.size):
        e = np.zeros(x.size)
        e[flat] = h
        e = e.reshape(x.shape)
        fd = (L(x + e, g, b) - L(x - e, g, b)) / (2 * h)
        assert abs(fd - dx.reshape(-1)[flat]) <= 1e-6 * max(1.0, abs(fd)), flat
    for c in range(C):
        e = np.zeros(C)
        e[c] = h
        assert abs((L(x, g + e, b) - L(x, g - e, b)) / (2 * h) - dgamma[c]) <= 1e-6 * max(1.0, abs(dgamma[c]))
        assert abs((L(x, g, b + e) - L(x, g, b - e)) / (2 * h) - dbeta[c]) <= 1e-6 * max(1.0, abs(dbeta[c]))


def test_bn_backward_is_linear_in_dy_and_scales_with_gamma():
    x, dy1, dy2, g = rnd(2, 3, 4, 4), rnd(2, 3, 4, 4), rnd(2, 3, 4, 4), rnd(3)
    a = ref.batchnorm2d_bwd(x, dy1, g, 1e-5)
    b = ref.batchnorm2d_bwd(x, dy2, g, 1e-5)
    c = ref.batchnorm2d_bwd(x, 2.0 * dy1 - 3.0 * dy2, g, 1e-5)
    for u, v, t in zip(a, b, c):
        assert np.max(np.abs(2.0 * u - 3.0 * v - t)) <= 1e-11
    d = ref.batchnorm2d_bwd(x, dy1, 2.0 * g, 1e-5)
    assert np.max(np.abs(d[0] - 2.0 * a[0])) <= 1e-12             # dx scales with gamma, dgamma and dbeta do not
    assert np.array_equal(d[1], a[1]) and np.array_equal(d[2], a[2])


def test_bn_rejects_bad_arguments():
    with pytest.raises(ValueError):
        ref.batchnorm2d_fwd(rnd(1, 1, 2, 2), np.ones(1), np.zeros(1), -1.0)
