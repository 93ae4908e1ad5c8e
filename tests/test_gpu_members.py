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
    err = float(np.abs(y - y_ref).max())
    a = np.argmax(y, 1)
    strict = float((a == np.argmax(y_ref, 1)).mean())
    near = float((y_ref[np.arange(len(a)), a] >= y_ref.max(1) - TOL_BF16).mean())
    print("%s: max-abs prob err %.3e, top-1 strict %.4f, in tolerance band %.4f" % (label, err, strict, near))
    assert np.isfinite(y).all()
    np.testing.assert_allclose(y.sum(1), 1.0, atol=1e-4)
    assert err <= TOL_BF16, (label, err)
    assert near >= TOP1, (label, near)
    return err, strict


SMALL = [
    ("resnet18", lambda: N.resnet18(size=64, classes=200), 64),
    ("resnet50", lambda: N.resnet50(size=64, classes=200), 64),
    ("densenet121", lambda: N.densenet121(size=64, classes=200), 64),
    ("efficientnet_b0", lambda: N.efficientnet(0, size=64, classes=200), 64),
    ("efficientnet_b2", lambda: N.efficientnet(2, size=64, classes=200), 64),
    ("inception_v3", lambda: N.inception_v3(size=107, classes=200), 107),
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
