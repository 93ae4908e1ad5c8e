"""Parity of whole members and of the heterogeneous ensembles against the CPU oracle.

Every member family (residual, dense, inception, inverted-residual) is run through the C interface
at a reduced input size the oracle finishes in seconds, then the heterogeneous and the heavy
ensemble are run at their full sizes on a few images.  bf16 members: combined probabilities within
2e-2, top-1 agreement >= 99.5 %, logits within a few percent of their spread.
"""
import numpy as np
import pytest

import oracle
import synth
from synth import nets as N
from synth import weights as W

pytestmark = pytest.mark.gpu
TOL_BF16, TOP1 = 2e-2, 0.995


@pytest.fixture(scope="module")
def ens():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2208_14049_amd as e
    e.lib()
    return e


def prepared(nets, seed, n, size):
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, seed, i)) for i, net in enumerate(nets)]
    imgs = W.make_images(seed + 1000, n, size, size)
    imgs[n // 2:] = W.make_images(seed + 1000, n - n // 2, size, size, first=n // 2, varied=True)
    return blobs, W.round_bf16(imgs)


def check(y, y_ref, label):
    """Probabilities within 2e-2; top-1 agreement >= 99.5 % up to ties inside that tolerance (the GPU's
    arg-max has an oracle probability within 2e-2 of the oracle's maximum), and strictly: a request of
    fewer than 200 images may hold one image whose arg-max differs (one of 256 is what the full-size
    requests of tests/test_gpu_full_size.py show for bf16 members: 99.6 %)."""
    err = float(np.abs(y - y_ref).max())
    a = np.argmax(y, 1)
    agree = a == np.argmax(y_ref, 1)
    strict = float(agree.mean())
    near = float((y_ref[np.arange(len(a)), a] >= y_ref.max(1) - TOL_BF16).mean())
    print("%s: max-abs prob err %.3e, top-1 strict %.4f, in tolerance band %.4f" % (label, err, strict, near))
    assert np.isfinite(y).all()
    np.testing.assert_allclose(y.sum(1), 1.0, atol=1e-4)
    assert err <= TOL_BF16, (label, err)
    assert near >= TOP1, (label, near)
    assert strict >= TOP1 or int((~agree).sum()) <= 1, (label, strict)
    return err, strict


SMALL = [
    ("resnet18", lambda: N.resnet18(size=64, classes=200), 64),
    ("resnet50", lambda: N.resnet50(size=64, classes=200), 64),
    ("densenet121", lambda: N.densenet121(size=64, classes=200), 64),
    ("efficientnet_b0", lambda: N.efficientnet(0, size=64, classes=200), 64),
    ("efficientnet_b2", lambda: N.efficientnet(2, size=64, classes=200), 64),
    ("inception_v3", lambda: N.inception_v3(size=107, classes=200), 107),
    ("resnext50", lambda: N.resnext50(size=64, classes=200), 64),
    ("vgg16", lambda: N.vgg(16, size=64, classes=200), 64),
    ("xception", lambda: N.xception(size=107, classes=200), 107),
    ("mobilenet_v2", lambda: N.mobilenet_v2(size=64, classes=200), 64),
]


@pytest.mark.parametrize("name,make,size", SMALL, ids=[s[0] for s in SMALL])
def test_member_family_small(ens, name, make, size):
    net = make()
    n = 11
    blobs, imgs = prepared([net], synth.BASE_SEED + 7, n, size)
    E = ens.Ensemble([net], blobs)
    E.ens_set_alloc([[4]])                                # batches of 4, 4, 3
    y = E.ens_predict(imgs)
    z = E.ens_member_logits(0, n)
    E.close()
    z_ref = oracle.forward_logits(net, blobs[0], imgs, real="f32")
    y_ref = oracle.softmax(z_ref.astype(np.float32), dtype=np.float32)
    rel = float(np.abs(z - z_ref).max() / z_ref.std())
    print("%s: logits max-abs err / logit std = %.4f (std %.3f)" % (name, rel, z_ref.std()))
    assert rel <= 0.08, (name, rel)
    check(y, y_ref, name)


def test_config3_heterogeneous_full_size(ens):
    """ResNet-50 (224), Inception-v3-shaped (299, fed by the library's resize), EfficientNet-B0-shaped,
    DenseNet-121-shaped; batch sizes differ per member, as a planner would choose them."""
    nets = N.config_members(3)
    n = 12
    blobs, imgs = prepared(nets, synth.BASE_SEED, n, 224)
    y_ref, _ = oracle.ensemble_predict(nets, blobs, imgs, real="f32")
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[8, 16, 32, 8]])
    y = E.ens_predict(imgs)
    check(y, y_ref, "config 3")
    E.ens_set_alloc([[8, 8, 8, 8], [0, 8, 0, 16]])        # a second worker for two of the members
    y2 = E.ens_predict(imgs)
    assert np.abs(y2 - y).max() <= 5e-3
    E.close()


def test_config6_vgg_xception_mobilenet_full_size(ens):
    """VGG-16-, Xception- (299, fed by the library's resize) and MobileNetV2-shaped members at their full
    sizes on a few images: the 7x7x512 -> 4096 layer of VGG (K = 25088), 728-channel separable blocks."""
    nets = [N.vgg(16), N.xception(size=299), N.mobilenet_v2()]
    n = 3
    blobs, imgs = prepared(nets, synth.BASE_SEED + 23, n, 224)
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[2, 2, 2]])
    y = E.ens_predict(imgs)
    E.close()
    y_ref, _ = oracle.ensemble_predict(nets, blobs, imgs, real="f32")
    check(y, y_ref, "config 6")


def test_config4_heavy_ensemble_full_size(ens):
    """Twelve members co-located on the one GPU, placed by worst-fit-decreasing."""
    nets = N.config_members(4)
    n = 4
    blobs, imgs = prepared(nets, synth.BASE_SEED, n, 224)
    y_ref, _ = oracle.ensemble_predict(nets, blobs, imgs, real="f32")
    E = ens.Ensemble(nets, blobs)
    out = E.ens_plan(0, strategy=1, n_calib=64, repeats=1)      # Algorithm 1 only
    assert out.matrix() == [[8] * 12] and out.score > 0
    y = E.ens_predict(imgs)
    check(y, y_ref, "config 4")
    E.close()


def test_config5_data_parallel_instances(ens):
    """One ResNet-50 served by k workers on separate streams: same predictions for every k and b."""
    nets = N.config_members(5)
    n = 40
    blobs, imgs = prepared(nets, synth.BASE_SEED, n, 224)
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[16]])
    y1 = E.ens_predict(imgs)
    z_ref = oracle.forward_logits(nets[0], blobs[0], imgs[:6], real="f32")
    check(y1[:6], oracle.softmax(z_ref.astype(np.float32), dtype=np.float32), "config 5")
    for k, b, seg in ((2, 4, 8), (4, 1, 4), (8, 16, 16), (1, 256, 256)):
        E.ens_set_alloc([[b]] * k, seg)
        y = E.ens_predict(imgs)
        assert np.abs(y - y1).max() <= 5e-3, (k, b)   # tile and K-split choice follow the batch size: fp32 sums in another order
    E.close()


def test_planner_on_the_gpu(ens):
    """Algorithm 1 + Algorithm 2 with real benchmarks on a small ensemble: the result is a valid
    matrix that fits the budget, is never slower than the start, and predicts the same values."""
    nets = [N.resnet18(size=64, classes=100), N.efficientnet(0, size=64, classes=100)]
    blobs, imgs = prepared(nets, 5, 64, 64)
    y_ref, _ = oracle.ensemble_predict(nets, blobs, imgs[:16], real="f32")
    E = ens.Ensemble(nets, blobs)
    start = E.ens_plan(0, strategy=1, n_calib=256, repeats=2)
    assert start.matrix() == [[8, 8], [0, 0]] or start.matrix() == [[8, 8]]
    out = E.ens_plan(0, strategy=0, slots=2, max_iter=3, max_neighs=8, n_calib=256, repeats=2, seed=3)
    A = out.matrix()
    assert len(A) == 2 and all(any(A[r][c] for r in range(2)) for c in range(2))
    assert all(v in (0, 8, 16, 32, 64, 128) for row in A for v in row)
    assert 1 <= out.n_bench <= 1 + 8 * 4 and out.score > 0
    y = E.ens_predict(imgs[:16])
    check(y, y_ref, "planned allocation")
    bbs = E.ens_plan(0, strategy=2, n_calib=256, repeats=2)
    assert bbs.n_bench == 10 and len(bbs.matrix()) == 1 and bbs.score > 0
    E.close()


# --------------------------------------------------------------------------- other combination rules
def _member_logits_oracle(nets, blobs, imgs):
    return [oracle.forward_logits(net, blob, oracle.resize_bilinear(imgs, net.in_h, net.in_w), real="f32")
            for net, blob in zip(nets, blobs)]


def test_weighted_average_and_vote_fp32(ens):
    """Weighted averaging and majority voting (section "The prediction accumulator") on config 1,
    fp32: weighted within 1e-4; votes exact wherever no member's top two logits are closer than the
    logit error of the fp32 path (both sides take the arg-max in fp32)."""
    nets = N.config_members(1)
    blobs = [W.make_blob(net, synth.BASE_SEED, i) for i, net in enumerate(nets)]
    imgs = W.make_images(synth.BASE_SEED + 1000, 200, 32, 32)
    imgs[100:] = W.make_images(synth.BASE_SEED + 1000, 100, 32, 32, first=100, varied=True)
    z = _member_logits_oracle(nets, blobs, imgs)
    probs = [oracle.softmax(v.astype(np.float32), dtype=np.float32) for v in z]
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[8, 8]])
    w = [0.3, 0.7]
    E.ens_set_combination("weighted", w)
    y = E.ens_predict(imgs)
    assert np.abs(y - oracle.combine_weighted(probs, w)).max() <= 1e-4
    assert np.abs(y.sum(1) - 1.0).max() <= 1e-5
    E.ens_set_combination("vote")
    y = E.ens_predict(imgs)
    ref = oracle.combine_vote(z)
    assert np.allclose(y.sum(1), 1.0, atol=1e-6)                 # M votes per sample
    assert set(np.unique(np.round(y * len(nets)).astype(int))) <= {0, 1, 2}
    clear = np.ones(len(imgs), bool)                             # samples where every member's arg-max is clear-cut
    for v in z:
        top2 = np.sort(v, axis=1)[:, -2:]
        clear &= (top2[:, 1] - top2[:, 0]) > 1e-4
    assert clear.mean() > 0.9
    assert np.array_equal(y[clear], ref[clear].astype(np.float32))
    # an ensemble of one under voting is the one-hot of its arg-max
    E.ens_set_combination("mean")
    y_mean = E.ens_predict(imgs)
    assert np.abs(y_mean - oracle.combine_mean(probs)).max() <= 1e-4
    with pytest.raises(Exception):
        E.ens_set_combination("weighted", None)
    E.close()


def test_vote_bf16_resnets(ens):
    """Majority voting over three bf16 ResNet-18-shaped members (1000 classes, batch 32): exact vote
    shares on the samples whose members' arg-max classes are clear of the bf16 logit error."""
    nets = N.config_members(2)
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, synth.BASE_SEED, i)) for i, net in enumerate(nets)]
    imgs = W.round_bf16(W.make_images(synth.BASE_SEED + 1000, 64, 224, 224, varied=True))
    z = _member_logits_oracle(nets, blobs, imgs)
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[32, 32, 32]])
    E.ens_set_combination("vote")
    y = E.ens_predict(imgs)
    zg = [E.ens_member_logits(m, len(imgs)) for m in range(3)]
    E.close()
    assert np.allclose(y.sum(1), 1.0, atol=1e-6)
    # the kernel's votes are exactly the arg-max of the logits the GPU itself produced ...
    assert np.array_equal(y, oracle.combine_vote(zg).astype(np.float32))
    # ... and agree with the oracle's wherever the oracle's top two logits differ by more than the bf16 path's error
    clear = np.ones(len(imgs), bool)
    for v, g in zip(z, zg):
        top2 = np.sort(v, axis=1)[:, -2:]
        clear &= (top2[:, 1] - top2[:, 0]) > 2.5 * np.abs(g - v).max()
    assert clear.sum() >= 8
    assert np.array_equal(y[clear], oracle.combine_vote(z)[clear].astype(np.float32))


def test_fake_predictor_overhead_run(ens):
    """The overhead experiment of section "Overhead of the inference system": with every forward
    pass replaced by zeros the accumulator still gathers all rows (softmax of zeros: uniform), and
    that run is a small fraction of the true one."""
    import time
    nets = N.config_members(2)
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, synth.BASE_SEED, i)) for i, net in enumerate(nets)]
    import torch
    imgs = torch.from_numpy(W.round_bf16(W.make_images(synth.BASE_SEED + 1000, 300, 224, 224))).cuda()
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[32, 32, 32], [32, 32, 32]])

    def run():
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        y = E.ens_predict(imgs)
        torch.cuda.synchronize()
        return y.cpu().numpy(), time.perf_counter() - t0
    y_true, _ = run()
    _, t_true = run()
    E.ens_debug_fake_predictor(1)
    y, _ = run()
    _, t_fake = run()
    assert np.allclose(y, 1.0 / 1000, atol=1e-7)                 # every row was gathered
    E.ens_debug_fake_predictor(0)
    assert np.array_equal(run()[0], y_true)                      # and the true path is back, bit for bit
    E.close()
    assert t_fake < 0.25 * t_true, (t_fake, t_true)
