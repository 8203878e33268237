"""Pins for the fp64 CPU oracle (no GPU).

None of these checks re-uses the oracle's own formulas: they are hand-worked
cases, closed forms, algebraic invariants, a brute-force evaluation written in
a different form (explicit zero padding + window slicing), and agreement with
an independent library's fp64 operators.  The paper itself prints no numbers
for these operators, so the definitions are the textbook ones of the network it
names as its benchmark ("GPU Speedup Analysis", "Simulation Results").
"""
import json
import os

import numpy as np
import pytest

import oracle
from workloads import (BN_EPS, CONV_SPECS, STAGE_IO, conv_out_hw, make_input,
                       make_resnet18_params)

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")))
RNG = np.random.default_rng(1234)


def a4(x):
    return np.asarray(x, dtype=np.float64)[None, None]


# ---------------------------------------------------------------- hand cases
def test_conv_hand_ones():
    g = GOLD["conv_ones_3x3_s1_p1"]
    y = oracle.conv2d(a4(g["x"]), np.ones((1, 1, 3, 3)), 1, 1)
    assert np.array_equal(y[0, 0], np.asarray(g["y"], dtype=np.float64))


def test_conv_hand_delta_is_cross_correlation():
    g = GOLD["conv_delta_at_00_s1_p1"]
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 0] = 1
    y = oracle.conv2d(a4(g["x"]), w, 1, 1)
    assert np.array_equal(y[0, 0], np.asarray(g["y"], dtype=np.float64))


def test_conv_hand_stride2():
    g = GOLD["conv_ones_3x3_s2_p1_on_4x4"]
    y = oracle.conv2d(a4(g["x"]), np.ones((1, 1, 3, 3)), 2, 1)
    assert np.array_equal(y[0, 0], np.asarray(g["y"], dtype=np.float64))


def test_maxpool_hand_negative_padding_never_wins():
    g = GOLD["maxpool_3x3_s2_p1_negative_4x4"]
    y = oracle.maxpool2d(a4(g["x"]), 3, 2, 1)
    assert np.array_equal(y[0, 0], np.asarray(g["y"], dtype=np.float64))


def test_bn_hand():
    g = GOLD["bn_scalar"]
    eps = 1e-5
    var = g["var_plus_eps"] - eps
    x = np.full((1, 1, 1, 1), g["x"])
    y = oracle.bn(x, [g["gamma"]], [g["beta"]], [g["mean"]], [var], eps)
    assert abs(y.item() - g["y"]) < 1e-12
    sc, sh = oracle.bn_fold([g["gamma"]], [g["beta"]], [g["mean"]], [var], eps)
    assert abs(sc[0] - g["scale"]) < 1e-12 and abs(sh[0] - g["shift"]) < 1e-12
    assert abs(oracle.scale_shift(x, sc, sh).item() - g["y"]) < 1e-12


def test_avgpool_fc_hand():
    g = GOLD["avgpool_fc"]
    x = np.asarray(g["x"], dtype=np.float64)[None]
    v = oracle.global_avgpool(x)
    assert np.allclose(v[0], g["v"], atol=1e-15)
    y = oracle.fc(v, g["w"], g["b"])
    assert np.allclose(y[0], g["y"], atol=1e-15)
    assert np.allclose(oracle.fc(v, g["w"], None)[0], np.asarray(g["y"]) - np.asarray(g["b"]))


def test_basic_block_hand_delta_identity_bn():
    # centre-delta kernels on the channel diagonal + identity BN:
    # out = ReLU(ReLU(x) + x) = 2x for x >= 0 and 0 for x < 0
    C, H = 3, 5
    x = RNG.standard_normal((2, C, H, H))
    w = np.zeros((C, C, 3, 3))
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    ident = (np.ones(C), np.zeros(C), np.zeros(C), np.full(C, 1.0 - BN_EPS))
    y = oracle.basic_block(x, [(w,) + ident, (w,) + ident], BN_EPS, 1)
    assert np.allclose(y, np.where(x >= 0, 2 * x, 0.0), atol=1e-12)


def test_out_size_closed_form():
    assert oracle.out_size(224, 7, 2, 3) == 112
    assert oracle.out_size(112, 3, 2, 1) == 56
    assert oracle.out_size(56, 3, 1, 1) == 56
    assert oracle.out_size(56, 1, 2, 0) == 28
    assert oracle.out_size(7, 3, 1, 1) == 7
    assert oracle.out_size(5, 3, 2, 1) == 3  # floor((5+2-3)/2)+1


# ---------------------------------------------------------------- brute force
def brute_conv(x, w, stride, pad):
    """Explicit zero padding, then one window product per output element."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    y = np.zeros((N, K, P, Q))
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    win = xp[n, :, p * stride:p * stride + R, q * stride:q * stride + S]
                    y[n, k, p, q] = float(np.sum(win * w[k]))
    return y


@pytest.mark.parametrize("C,K,H,W,R,stride,pad", [
    (3, 4, 9, 7, 3, 1, 1), (2, 3, 8, 10, 3, 2, 1), (3, 2, 12, 11, 7, 2, 3), (4, 5, 6, 6, 1, 2, 0),
    (1, 1, 5, 5, 3, 1, 0), (2, 2, 7, 9, 5, 3, 2),
])
def test_conv_brute_force(C, K, H, W, R, stride, pad):
    x = RNG.standard_normal((2, C, H, W))
    w = RNG.standard_normal((K, C, R, R))
    assert np.allclose(oracle.conv2d(x, w, stride, pad), brute_conv(x, w, stride, pad),
                       rtol=0, atol=1e-12)


def test_maxpool_brute_force():
    x = RNG.standard_normal((2, 3, 9, 11))
    xp = np.full((2, 3, 11, 13), -np.inf)
    xp[:, :, 1:10, 1:12] = x
    P, Q = (9 + 2 - 3) // 2 + 1, (11 + 2 - 3) // 2 + 1
    ref = np.empty((2, 3, P, Q))
    for p in range(P):
        for q in range(Q):
            ref[:, :, p, q] = xp[:, :, 2 * p:2 * p + 3, 2 * q:2 * q + 3].max(axis=(2, 3))
    assert np.array_equal(oracle.maxpool2d(x, 3, 2, 1), ref)


# ---------------------------------------------------------------- invariants
def test_conv_centre_delta_is_identity_multichannel():
    C = 5
    x = RNG.standard_normal((2, C, 7, 6))
    w = np.zeros((C, C, 3, 3))
    w[np.arange(C), np.arange(C), 1, 1] = 1
    assert np.array_equal(oracle.conv2d(x, w, 1, 1), x)


def test_conv_linearity_in_x_and_w():
    x1, x2 = RNG.standard_normal((2, 1, 3, 8, 8))
    w1, w2 = RNG.standard_normal((2, 4, 3, 3, 3))
    a, b = 0.7, -1.3
    f = lambda x, w: oracle.conv2d(x, w, 2, 1)
    assert np.allclose(f(a * x1 + b * x2, w1), a * f(x1, w1) + b * f(x2, w1), atol=1e-12)
    assert np.allclose(f(x1, a * w1 + b * w2), a * f(x1, w1) + b * f(x1, w2), atol=1e-12)


def test_conv_all_ones_counts_valid_taps():
    C, H = 4, 6
    y = oracle.conv2d(np.ones((1, C, H, H)), np.ones((2, C, 3, 3)), 1, 1)
    cnt = np.full((H, H), 9.0)
    cnt[0, :] = cnt[-1, :] = cnt[:, 0] = cnt[:, -1] = 6
    cnt[0, 0] = cnt[0, -1] = cnt[-1, 0] = cnt[-1, -1] = 4
    assert np.array_equal(y[0, 0], C * cnt) and np.array_equal(y[0, 1], C * cnt)


def test_conv_1x1_is_per_pixel_matrix_product():
    x = RNG.standard_normal((2, 6, 8, 8))
    w = RNG.standard_normal((5, 6, 1, 1))
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x[:, :, ::2, ::2])
    assert np.allclose(oracle.conv2d(x, w, 2, 0), ref, atol=1e-12)


def test_conv_full_kernel_is_dot_product_and_equals_fc():
    x = RNG.standard_normal((3, 4, 5, 5))
    w = RNG.standard_normal((7, 4, 5, 5))
    y = oracle.conv2d(x, w, 1, 0)
    assert y.shape == (3, 7, 1, 1)
    ref = x.reshape(3, -1) @ w.reshape(7, -1).T
    assert np.allclose(y[:, :, 0, 0], ref, atol=1e-12)
    assert np.allclose(oracle.fc(x.reshape(3, -1), w.reshape(7, -1)), ref, atol=1e-12)


def test_conv_translation_equivariance_interior():
    x = np.zeros((1, 2, 12, 12))
    x[:, :, 3:7, 3:7] = RNG.standard_normal((1, 2, 4, 4))
    xs = np.roll(x, (2, 3), axis=(2, 3))
    w = RNG.standard_normal((3, 2, 3, 3))
    assert np.allclose(np.roll(oracle.conv2d(x, w, 1, 1), (2, 3), axis=(2, 3)),
                       oracle.conv2d(xs, w, 1, 1), atol=1e-12)


def test_conv_distinguishes_r_from_s_and_k_from_c():
    # a transposed kernel or swapped channel roles must change the answer
    x = RNG.standard_normal((1, 2, 6, 6))
    w = RNG.standard_normal((3, 2, 3, 3))
    y = oracle.conv2d(x, w, 1, 1)
    assert not np.allclose(y, oracle.conv2d(x, w.transpose(0, 1, 3, 2), 1, 1))
    ref = brute_conv(x, w, 1, 1)
    assert np.allclose(y, ref, atol=1e-12)


def test_maxpool_invariants():
    x = RNG.standard_normal((2, 3, 10, 10))
    d = np.abs(RNG.standard_normal(x.shape))
    p = oracle.maxpool2d(x)
    assert np.all(oracle.maxpool2d(x + d) >= p)                      # monotone
    assert np.array_equal(oracle.maxpool2d(np.full_like(x, -3.5)), np.full((2, 3, 5, 5), -3.5))
    assert np.allclose(oracle.maxpool2d(2.5 * x - 1.0), 2.5 * p - 1.0, atol=1e-12)  # increasing affine
    assert np.all(p >= x[:, :, ::2, ::2])                            # window centre is 2p,2q
    assert p.shape == (2, 3, 5, 5)


def test_avgpool_const_and_mean():
    assert np.allclose(oracle.global_avgpool(np.full((2, 3, 7, 7), 1.25)), 1.25)
    x = RNG.standard_normal((2, 3, 7, 7))
    assert np.allclose(oracle.global_avgpool(x), x.mean(axis=(2, 3)), atol=1e-14)


def test_bn_folded_equals_unfolded():
    C = 16
    x = RNG.standard_normal((2, C, 5, 5))
    g, b = RNG.uniform(0.5, 1.5, C), RNG.standard_normal(C) * 0.1
    m, v = RNG.standard_normal(C) * 0.1, RNG.uniform(0.5, 1.5, C)
    sc, sh = oracle.bn_fold(g, b, m, v, BN_EPS)
    assert np.allclose(oracle.bn(x, g, b, m, v, BN_EPS), oracle.scale_shift(x, sc, sh),
                       rtol=1e-13, atol=1e-13)
    # closed form on one element, typed independently
    ref = g[3] * (x[1, 3, 2, 2] - m[3]) / np.sqrt(v[3] + BN_EPS) + b[3]
    assert abs(oracle.bn(x, g, b, m, v, BN_EPS)[1, 3, 2, 2] - ref) < 1e-13


def test_relu_add():
    a, b = RNG.standard_normal((2, 50))
    assert np.array_equal(oracle.relu(a), np.maximum(a, 0))
    assert np.array_equal(oracle.add(a, b), a + b)


# ---------------------------------------------------------------- layer table
def test_layer_table_closed_forms():
    g = GOLD["resnet18_closed_forms"]
    macs = sum(conv_out_hw(h, k, s, p) ** 2 * co * ci * k * k for _, ci, co, k, s, p, h in CONV_SPECS)
    macs += 512 * 1000
    params = sum(co * ci * k * k + 2 * co for _, ci, co, k, _, _, _ in CONV_SPECS) + 512 * 1000 + 1000
    assert macs == g["macs_per_image"] and params == g["params"]
    assert len(CONV_SPECS) == 20 and len(STAGE_IO) == 6


# ---------------------------------------------------------------- library cross-check
torch = pytest.importorskip("torch")
F = torch.nn.functional


def t64(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))


@pytest.mark.parametrize("C,K,H,R,stride,pad", [(3, 8, 30, 7, 2, 3), (8, 8, 14, 3, 1, 1),
                                                (8, 16, 14, 3, 2, 1), (8, 16, 14, 1, 2, 0)])
def test_ops_against_library_fp64(C, K, H, R, stride, pad):
    x = RNG.standard_normal((2, C, H, H)); w = RNG.standard_normal((K, C, R, R))
    ref = F.conv2d(t64(x), t64(w), None, stride, pad).numpy()
    assert np.allclose(oracle.conv2d(x, w, stride, pad), ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(oracle.maxpool2d(x), F.max_pool2d(t64(x), 3, 2, 1).numpy())
    g, b = RNG.uniform(0.5, 1.5, C), RNG.standard_normal(C)
    m, v = RNG.standard_normal(C), RNG.uniform(0.5, 1.5, C)
    refbn = F.batch_norm(t64(x), t64(m), t64(v), t64(g), t64(b), False, 0.0, BN_EPS).numpy()
    assert np.allclose(oracle.bn(x, g, b, m, v, BN_EPS), refbn, rtol=1e-12, atol=1e-12)


def torch_resnet18(params, x, upto=6):
    """ResNet18 wired independently of the oracle, on the library's fp64 ops."""
    def cb(t, i, stride, pad, relu):
        t = F.conv2d(t, t64(params["conv_w"][i]), None, stride, pad)
        t = F.batch_norm(t, t64(params["mean"][i]), t64(params["var"][i]), t64(params["gamma"][i]),
                         t64(params["beta"][i]), False, 0.0, BN_EPS)
        return F.relu(t) if relu else t
    outs = []
    t = F.max_pool2d(cb(t64(x), 0, 2, 3, True), 3, 2, 1); outs.append(t)
    for i in (1, 3):
        t = F.relu(cb(cb(t, i, 1, 1, True), i + 1, 1, 1, False) + t)
    outs.append(t)
    for first in (5, 10, 15):
        sc = cb(t, first + 2, 2, 0, False)
        t = F.relu(cb(cb(t, first, 2, 1, True), first + 1, 1, 1, False) + sc)
        t = F.relu(cb(cb(t, first + 3, 1, 1, True), first + 4, 1, 1, False) + t)
        outs.append(t)
    v = t.mean(dim=(2, 3))
    outs.append(F.linear(v, t64(params["fc_w"]), t64(params["fc_b"])))
    return [o.numpy() for o in outs]


@pytest.fixture(scope="module")
def net():
    params = make_resnet18_params(1, 0)
    x = make_input(1, 0, (2, 3, 224, 224))
    logits, outs = oracle.resnet18(params, BN_EPS, x, want_stages=True)
    return params, x, logits, outs


def test_resnet18_against_library_wiring(net):
    params, x, logits, outs = net
    ref = torch_resnet18(params, x)
    for j in range(6):
        assert outs[j].shape == ref[j].shape
        assert np.allclose(outs[j], ref[j], rtol=1e-10, atol=1e-10), j
    assert np.array_equal(outs[5], logits)
    assert np.array_equal(np.argmax(logits, 1), np.argmax(ref[5], 1))


def test_stage_composition_and_batch_independence(net):
    params, x, logits, outs = net
    # stages chained one by one == whole network
    t = x
    for j in range(6):
        t = oracle.resnet18_stage(j, params, BN_EPS, t)
        assert np.array_equal(t, outs[j])
    # image 1 alone == row 1 of the batch
    l1 = oracle.resnet18(params, BN_EPS, x[1:2])
    assert np.array_equal(l1[0], logits[1])
    for j, ((ci, hi, wi), (co, ho, wo)) in enumerate(STAGE_IO):
        assert outs[j].shape[1:] == ((co,) if j == 5 else (co, ho, wo))
    with pytest.raises(ValueError):
        oracle.resnet18_stage(6, params, BN_EPS, x)


def test_block_with_projection_against_library():
    C, K, H = 4, 8, 10
    x = RNG.standard_normal((2, C, H, H))
    def mk(co, ci, k):
        return (RNG.standard_normal((co, ci, k, k)), RNG.uniform(0.5, 1.5, co),
                RNG.standard_normal(co) * 0.1, RNG.standard_normal(co) * 0.1,
                RNG.uniform(0.5, 1.5, co))
    c1, c2, cd = mk(K, C, 3), mk(K, K, 3), mk(K, C, 1)
    y = oracle.basic_block(x, [c1, c2, cd], BN_EPS, 2)
    def cb(t, p, stride, pad):
        t = F.conv2d(t, t64(p[0]), None, stride, pad)
        return F.batch_norm(t, t64(p[3]), t64(p[4]), t64(p[1]), t64(p[2]), False, 0.0, BN_EPS)
    ref = F.relu(cb(F.relu(cb(t64(x), c1, 2, 1)), c2, 1, 1) + cb(t64(x), cd, 2, 0)).numpy()
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-11)
