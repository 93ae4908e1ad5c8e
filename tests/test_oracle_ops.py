"""Pins of the forward-pass oracle against facts that do not come from the oracle:
closed forms, identities, and PyTorch's CPU library routines in fp64."""
import numpy as np
import pytest

import oracle
import synth
from synth import nets as N
from synth import weights as W
from tests import torch_ref

RNG = np.random.default_rng(7)


def one_conv(h, w, cin, cout, k, stride=1, pad="same", **kw):
    n = N.Net("t", h, w, 1, dtype="fp32", in_c=cin)
    t = n.conv(0, cout, k, stride=stride, pad=pad, **kw)
    n.out_tensor = t
    return n


def run_oracle(net, blob, x, real="f64"):
    out = oracle.forward_logits(net, blob, x, real=real)
    h, w, c = net.tensors[net.out_tensor]
    return out.reshape(x.shape[0], h, w, c)


def set_w(net, blob, arr, which=0):
    p = [p for p in net.params if p["role"] == "conv_w"][which]
    blob[p["offset"]:p["offset"] + p["size"]] = np.asarray(arr, dtype=np.float32).ravel()


# ---------------------------------------------------------------- convolution
@pytest.mark.parametrize("k", [1, 3, 5, 7, (1, 7), (7, 1), (1, 3), (3, 1)])
def test_delta_kernel_is_identity(k):
    kh, kw = (k, k) if isinstance(k, int) else k
    c = 4
    net = one_conv(9, 11, c, c, k, bn=False, act=None, bias=False)
    blob = np.zeros(net.blob_size, np.float32)
    w = np.zeros((kh, kw, c, c), np.float32)
    w[kh // 2, kw // 2] = np.eye(c)
    set_w(net, blob, w)
    x = RNG.standard_normal((2, 9, 11, c)).astype(np.float32)
    assert np.array_equal(run_oracle(net, blob, x), x.astype(np.float64))


@pytest.mark.parametrize("k,tap", [(3, (0, 0)), (3, (2, 1)), (5, (4, 0)), ((1, 7), (0, 6)), ((7, 1), (1, 0))])
def test_shifted_delta_shifts_with_zero_fill(k, tap):
    kh, kw = (k, k) if isinstance(k, int) else k
    c = 3
    net = one_conv(8, 10, c, c, k, bn=False, act=None, bias=False)
    blob = np.zeros(net.blob_size, np.float32)
    w = np.zeros((kh, kw, c, c), np.float32)
    w[tap[0], tap[1]] = np.eye(c)
    set_w(net, blob, w)
    x = RNG.standard_normal((1, 8, 10, c)).astype(np.float32)
    y = run_oracle(net, blob, x)
    dh, dw = tap[0] - (kh - 1) // 2, tap[1] - (kw - 1) // 2
    exp = np.zeros_like(y)
    for ho in range(8):
        for wo in range(10):
            hi, wi = ho + dh, wo + dw
            if 0 <= hi < 8 and 0 <= wi < 10:
                exp[0, ho, wo] = x[0, hi, wi]
    assert np.array_equal(y, exp)


@pytest.mark.parametrize("k", [3, 5, 7])
def test_all_ones_counts_window_overlap(k):
    cin = 2
    net = one_conv(6, 7, cin, 1, k, bn=False, act=None, bias=False)
    blob = np.ones(net.blob_size, np.float32)
    x = np.ones((1, 6, 7, cin), np.float32)
    y = run_oracle(net, blob, x)[0, :, :, 0]
    p = (k - 1) // 2
    for ho in range(6):
        for wo in range(7):
            nh = min(ho + p, 5) - max(ho - p, 0) + 1
            nw = min(wo + p, 6) - max(wo - p, 0) + 1
            assert y[ho, wo] == nh * nw * cin


def test_1x1_is_matrix_product():
    net = one_conv(5, 6, 7, 9, 1, bn=False, act=None, bias=False)
    blob = W.make_blob(net, 1, 0)
    x = RNG.standard_normal((3, 5, 6, 7)).astype(np.float32)
    w = blob[:63].astype(np.float64).reshape(7, 9)
    exp = x.astype(np.float64).reshape(-1, 7) @ w
    np.testing.assert_allclose(run_oracle(net, blob, x).reshape(-1, 9), exp, rtol=1e-12, atol=1e-12)


def test_stride2_is_subsampled_stride1():
    n1 = one_conv(12, 12, 3, 5, 3, stride=1, bn=False, act=None, bias=False)
    n2 = one_conv(12, 12, 3, 5, 3, stride=2, bn=False, act=None, bias=False)
    blob = W.make_blob(n1, 2, 0)
    x = RNG.standard_normal((2, 12, 12, 3)).astype(np.float32)
    y1, y2 = run_oracle(n1, blob, x), run_oracle(n2, blob, x)
    assert y2.shape == (2, 6, 6, 5)
    assert np.array_equal(y2, y1[:, ::2, ::2])


def test_brute_force_seven_loops_tiny():
    net = one_conv(5, 5, 3, 4, 3, stride=2, bn=False, act=None, bias=True)
    blob = W.make_blob(net, 3, 0)
    x = RNG.standard_normal((2, 5, 5, 3)).astype(np.float32)
    w = blob[:108].astype(np.float64).reshape(3, 3, 3, 4)
    b = blob[108:112].astype(np.float64)
    exp = np.zeros((2, 3, 3, 4))
    for i in range(2):
        for ho in range(3):
            for wo in range(3):
                for co in range(4):
                    s = b[co]
                    for kh in range(3):
                        for kw in range(3):
                            for ci in range(3):
                                hi, wi = ho * 2 - 1 + kh, wo * 2 - 1 + kw
                                if 0 <= hi < 5 and 0 <= wi < 5:
                                    s += float(x[i, hi, wi, ci]) * w[kh, kw, ci, co]
                    exp[i, ho, wo, co] = s
    np.testing.assert_allclose(run_oracle(net, blob, x), exp, rtol=1e-12, atol=1e-13)


CONV_CASES = [
    dict(k=1, stride=1), dict(k=1, stride=2), dict(k=3, stride=1), dict(k=3, stride=2),
    dict(k=5, stride=1), dict(k=5, stride=2), dict(k=7, stride=2), dict(k=(1, 7)), dict(k=(7, 1)),
    dict(k=(1, 3)), dict(k=(3, 1)), dict(k=3, stride=2, pad="valid"), dict(k=3, pad="valid"),
    dict(k=3, act="silu"), dict(k=3, bn=False), dict(k=1, pre=True), dict(k=3, pre=True),
    dict(k=3, groups=2), dict(k=3, stride=2, groups=2), dict(k=1, groups=2, bn=False),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: str(c))
def test_conv_against_library_conv2d(case):
    net = one_conv(13, 10, 6, 8, **case)
    blob = W.make_blob(net, 5, 0)
    x = RNG.standard_normal((2, 13, 10, 6)).astype(np.float32)
    got = run_oracle(net, blob, x)
    exp = torch_ref.run(net, blob, x, want=net.out_tensor)
    np.testing.assert_allclose(got, exp, rtol=1e-11, atol=1e-11)


def test_grouped_conv_is_independent_convs_on_channel_slices():
    """A convolution with g groups equals g ordinary convolutions, group j reading input channels
    [j*cin/g, (j+1)*cin/g) and writing output channels [j*cout/g, (j+1)*cout/g) with columns
    [j*cout/g, (j+1)*cout/g) of the [kh][kw][cin/g][cout] weights (the definition of groups)."""
    g, cin, cout = 3, 6, 12
    a = N.Net("g", 7, 9, 1, dtype="fp32", in_c=cin)
    a.out_tensor = a.conv(0, cout, 3, bn=False, act=None, bias=True, groups=g)
    blob = W.make_blob(a, 9, 0)
    x = RNG.standard_normal((2, 7, 9, cin)).astype(np.float32)
    got = run_oracle(a, blob, x)
    w = blob[:9 * (cin // g) * cout].reshape(3, 3, cin // g, cout)
    bias = blob[9 * (cin // g) * cout:9 * (cin // g) * cout + cout]
    for j in range(g):
        b = N.Net("s", 7, 9, 1, dtype="fp32", in_c=cin // g)
        b.out_tensor = b.conv(0, cout // g, 3, bn=False, act=None, bias=True)
        bb = np.concatenate([w[..., j * (cout // g):(j + 1) * (cout // g)].ravel(),
                             bias[j * (cout // g):(j + 1) * (cout // g)]]).astype(np.float32)
        exp = run_oracle(b, bb, x[..., j * (cin // g):(j + 1) * (cin // g)])
        np.testing.assert_allclose(got[..., j * (cout // g):(j + 1) * (cout // g)], exp, rtol=1e-12, atol=1e-12)
    # and a group never sees another group's input
    x2 = x.copy()
    x2[..., :cin // g] += 5.0
    got2 = run_oracle(a, blob, x2)
    assert np.all(got2[..., cout // g:] == got[..., cout // g:]) and not np.allclose(got2[..., :cout // g], got[..., :cout // g])


def test_conv_channel_slices_and_residual():
    n = N.Net("t", 8, 8, 1, dtype="fp32", in_c=12)
    o = n.tensor(8, 8, 20)
    n.conv(0, 6, 3, src_slice=(4, 5), dst=(o, 2))
    n.conv(0, 6, 1, src_slice=(0, 12), dst=(o, 10), res=(o, 2), act="relu")
    n.out_tensor = o
    blob = W.make_blob(n, 6, 0)
    x = RNG.standard_normal((2, 8, 8, 12)).astype(np.float32)
    got = run_oracle(n, blob, x)
    exp = torch_ref.run(n, blob, x, want=o)
    np.testing.assert_allclose(got, exp, rtol=1e-11, atol=1e-11)
    assert np.all(got[..., :2] == 0) and np.all(got[..., 16:] == 0) and np.all(got[..., 8:10] == 0)


def test_bn_identity_parameters():
    net = one_conv(6, 6, 3, 3, 1, bn=True, act=None)
    blob = np.zeros(net.blob_size, np.float32)
    set_w(net, blob, np.eye(3).reshape(1, 1, 3, 3))
    bn = [p for p in net.params if p["role"] == "bn"][0]["offset"]
    blob[bn:bn + 3] = 1.0                        # gamma
    blob[bn + 9:bn + 12] = 1.0 - N.BN_EPS        # variance
    x = RNG.standard_normal((1, 6, 6, 3)).astype(np.float32)
    np.testing.assert_allclose(run_oracle(net, blob, x), x, rtol=0, atol=1e-7)


def test_bn_closed_form():
    net = one_conv(4, 4, 2, 2, 1, bn=True, act=None)
    blob = np.zeros(net.blob_size, np.float32)
    set_w(net, blob, np.eye(2).reshape(1, 1, 2, 2))
    bn = [p for p in net.params if p["role"] == "bn"][0]["offset"]
    blob[bn:bn + 8] = [2.0, 0.5, 0.25, -1.0, 1.0, -2.0, 4.0 - N.BN_EPS, 0.25 - N.BN_EPS]
    x = np.full((1, 4, 4, 2), 3.0, np.float32)
    y = run_oracle(net, blob, x)
    np.testing.assert_allclose(y[..., 0], 2.0 * (3.0 - 1.0) / 2.0 + 0.25, atol=1e-6)
    np.testing.assert_allclose(y[..., 1], 0.5 * (3.0 + 2.0) / 0.5 - 1.0, atol=1e-6)


# ---------------------------------------------------------------- depthwise
@pytest.mark.parametrize("k,stride", [(3, 1), (3, 2), (5, 1), (5, 2)])
def test_depthwise_equals_block_diagonal_dense_and_library(k, stride):
    c = 6
    nd = N.Net("d", 11, 9, 1, dtype="fp32", in_c=c)
    nd.out_tensor = nd.dwconv(0, k, stride, bn=True, act="silu")
    blob = W.make_blob(nd, 8, 0)
    x = RNG.standard_normal((2, 11, 9, c)).astype(np.float32)
    got = run_oracle(nd, blob, x)
    np.testing.assert_allclose(got, torch_ref.run(nd, blob, x, want=nd.out_tensor), rtol=1e-11, atol=1e-11)
    # same filter as a dense convolution whose weight is diagonal in (cin, cout)
    nc = one_conv(11, 9, c, c, k, stride=stride, bn=True, act="silu")
    blob2 = np.zeros(nc.blob_size, np.float32)
    wd = blob[:k * k * c].reshape(k, k, c)
    dense = np.zeros((k, k, c, c), np.float32)
    for ch in range(c):
        dense[:, :, ch, ch] = wd[:, :, ch]
    set_w(nc, blob2, dense)
    o1 = [p for p in nd.params if p["role"] == "bn"][0]["offset"]
    o2 = [p for p in nc.params if p["role"] == "bn"][0]["offset"]
    blob2[o2:o2 + 4 * c] = blob[o1:o1 + 4 * c]
    np.testing.assert_allclose(got, run_oracle(nc, blob2, x), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- squeeze-excite
def test_se_zero_weights_halves_input():
    n = N.Net("s", 5, 5, 1, dtype="fp32", in_c=8)
    n.out_tensor = n.se(0, 2)
    blob = np.zeros(n.blob_size, np.float32)
    x = RNG.standard_normal((2, 5, 5, 8)).astype(np.float32)
    assert np.array_equal(run_oracle(n, blob, x), 0.5 * x.astype(np.float64))


def test_se_against_library():
    n = N.Net("s", 7, 6, 1, dtype="fp32", in_c=16)
    n.out_tensor = n.se(0, 4)
    blob = W.make_blob(n, 9, 0)
    x = RNG.standard_normal((3, 7, 6, 16)).astype(np.float32)
    np.testing.assert_allclose(run_oracle(n, blob, x), torch_ref.run(n, blob, x, want=n.out_tensor),
                               rtol=1e-11, atol=1e-11)


# ---------------------------------------------------------------- pooling
@pytest.mark.parametrize("kind", ["max", "avg"])
@pytest.mark.parametrize("k,s,p", [(2, 2, 0), (3, 2, 1), (3, 1, 1), (3, 2, 0)])
def test_pool_constant_and_library(kind, k, s, p):
    n = N.Net("p", 9, 12, 1, dtype="fp32", in_c=3)
    n.out_tensor = (n.maxpool if kind == "max" else n.avgpool)(0, k, s, p)
    blob = np.zeros(0, np.float32)
    const = np.full((1, 9, 12, 3), -2.5, np.float32)
    assert np.all(run_oracle(n, blob, const) == -2.5)
    x = RNG.standard_normal((2, 9, 12, 3)).astype(np.float32)
    np.testing.assert_allclose(run_oracle(n, blob, x), torch_ref.run(n, blob, x, want=n.out_tensor),
                               rtol=1e-12, atol=1e-12)


def test_global_average_of_ramp():
    n = N.Net("g", 4, 5, 1, dtype="fp32", in_c=2)
    n.out_tensor = n.gap(0)
    x = np.zeros((1, 4, 5, 2), np.float32)
    x[0, :, :, 0] = np.arange(20).reshape(4, 5)
    x[0, :, :, 1] = 3.0
    y = run_oracle(n, np.zeros(0, np.float32), x)
    assert y.shape == (1, 1, 1, 2)
    np.testing.assert_allclose(y[0, 0, 0], [9.5, 3.0], rtol=1e-15)


def test_fc_is_matrix_product_plus_bias():
    n = N.Net("f", 1, 1, 5, dtype="fp32", in_c=7)
    n.fc(0, 5)
    blob = W.make_blob(n, 11, 0)
    x = RNG.standard_normal((4, 1, 1, 7)).astype(np.float32)
    exp = x.reshape(4, 7).astype(np.float64) @ blob[:35].astype(np.float64).reshape(7, 5) + blob[35:40]
    np.testing.assert_allclose(oracle.forward_logits(n, blob, x, real="f64"), exp, rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- whole members
def _small_members():
    return [
        N.tiny_a(), N.tiny_b(),
        N.resnet18(size=64, classes=17), N.resnet50(size=64, classes=17),
        N.densenet121(size=64, classes=17), N.efficientnet(0, size=64, classes=17),
        N.inception_v3(size=107, classes=17), N.resnext50(size=64, classes=17),
        N.xception(size=107, classes=17), N.mobilenet_v2(size=64, classes=17), N.vgg(16, size=64, classes=17),
    ]


@pytest.mark.parametrize("net", _small_members(), ids=lambda n: n.name)
def test_member_against_library_interpreter(net):
    blob = W.make_blob(net, synth.BASE_SEED, 3)
    x = W.make_images(synth.BASE_SEED + 1000, 2, net.in_h, net.in_w)
    got = oracle.forward_logits(net, blob, x, real="f64")
    exp = torch_ref.run(net, blob, x)
    assert np.isfinite(got).all() and got.std() > 1e-3
    np.testing.assert_allclose(got, exp, rtol=1e-9, atol=1e-9)
    got32 = oracle.forward_logits(net, blob, x, real="f32")
    np.testing.assert_allclose(got32, exp, rtol=0, atol=2e-4 * max(1.0, np.abs(exp).max()))


def test_architecture_work_matches_published_figures():
    """Multiply-accumulates and weight counts of the member shapes equal the
    figures published for these architectures."""
    gmac = {"resnet18": 1.814, "resnet34": 3.664, "resnet50": 4.089, "resnet101": 7.801,
            "resnet152": 11.514, "densenet121": 2.834, "densenet169": 3.360, "densenet201": 4.291}
    for name, g in gmac.items():
        net = getattr(N, name)()
        assert abs(net.macs() / 1e9 - g) < 2e-3, (name, net.macs())
    assert abs(N.resnet50().n_weights() / 1e6 - 25.5) < 0.1
    assert abs(N.resnet18().n_weights() / 1e6 - 11.7) < 0.1
    assert abs(N.efficientnet(0).macs() / 1e9 - 0.39) < 0.01
    assert abs(N.inception_v3().macs() / 1e9 - 5.7) < 0.05
    # VGG-16 / VGG-19: 15.5 / 19.6 GMAC, 138.4 / 143.7 M weights; Xception at 299: 8.4 GMAC, 22.9 M;
    # MobileNetV2: 0.30 GMAC, 3.5 M (the architecture papers' tables)
    assert abs(N.vgg(16).macs() / 1e9 - 15.47) < 0.02 and abs(N.vgg(16).n_weights() / 1e6 - 138.4) < 0.1
    assert abs(N.vgg(19).macs() / 1e9 - 19.63) < 0.02 and abs(N.vgg(19).n_weights() / 1e6 - 143.7) < 0.1
    assert abs(N.xception().macs() / 1e9 - 8.4) < 0.06 and abs(N.xception().n_weights() / 1e6 - 22.9) < 0.1
    assert abs(N.mobilenet_v2().macs() / 1e9 - 0.30) < 0.01 and abs(N.mobilenet_v2().n_weights() / 1e6 - 3.5) < 0.05
    # ResNeXt-50 (32x4d): 4.2 GMAC, 25.0 M weights
    assert abs(N.resnext50().macs() / 1e9 - 4.23) < 0.03 and abs(N.resnext50().n_weights() / 1e6 - 25.0) < 0.1


def test_bf16_storage_mode_brackets_fp32():
    net = N.resnet18(size=64, classes=50)
    blob = W.quantise_weights_bf16(net, W.make_blob(net, 4, 0))
    x = W.round_bf16(W.make_images(5, 4, 64, 64))
    a = oracle.forward_logits(net, blob, x)
    b = oracle.forward_logits(net, blob, x, store_bf16=True)
    err = np.abs(a - b).max()
    assert 0 < err < 0.05 * a.std() + 0.05
