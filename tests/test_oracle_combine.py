"""Pins of the combination-rule, partition and resize oracles."""
import json
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import synth
from synth import nets as N
from synth import weights as W

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))
RNG = np.random.default_rng(11)


def test_segments_worked_example():
    g = GOLD["segments_example"]
    segs = oracle.segments(g["nb_images"], g["segment_size"])
    assert [b - a for a, b in segs] == g["sizes"]
    assert segs[0][0] == 0 and segs[-1][1] == g["nb_images"]
    q = oracle.broadcast(g["nb_images"], g["segment_size"], g["n_models"])
    assert sum(len(v) for v in q.values()) == g["n_messages"]
    assert all(v == g["ids_per_queue"] for v in q.values())


@pytest.mark.parametrize("n,seg", [(0, 128), (1, 128), (128, 128), (129, 128), (1024, 128), (300, 7)])
def test_segments_cover_request_exactly_once(n, seg):
    segs = oracle.segments(n, seg)
    covered = [i for a, b in segs for i in range(a, b)]
    assert covered == list(range(n))
    assert all(b - a == seg for a, b in segs[:-1])
    for a, b in segs:
        for bs in (1, 8, 32, 128):
            bt = oracle.batches(a, b, bs)
            assert [i for x, y in bt for i in range(x, y)] == list(range(a, b))
            assert all(y - x == bs for x, y in bt[:-1]) and 0 < bt[-1][1] - bt[-1][0] <= bs


def test_fifo_hand_out_pins():
    """Workers of one DNN sharing a FIFO queue of segment ids (section "Data-parallelism"): every segment has
    exactly one owner; equal workers alternate; with no per-batch cost the batch size does not matter; a
    worker whose segments take half the time ends up with two thirds of them; the makespan is within one
    segment of the best possible split (the list-scheduling bound)."""
    assert oracle.fifo_hand_out(0, 128, [8, 8], 1.0, 1.0) == []
    assert oracle.fifo_hand_out(300, 128, [8], 1.0, 1.0) == [0, 0, 0]
    assert oracle.fifo_hand_out(128 * 7, 128, [32, 32, 32], 1e-3, 1e-5) == [0, 1, 2, 0, 1, 2, 0]
    assert oracle.fifo_hand_out(128 * 6, 128, [8, 128], 0.0, 1e-5) == [0, 1, 0, 1, 0, 1]
    # batch 64: 2 batches per segment, batch 128: 1; per-batch cost only -> worker 1 is twice as fast
    own = oracle.fifo_hand_out(128 * 300, 128, [64, 128], 1.0, 0.0)
    assert len(own) == 300 and abs(own.count(1) - 200) <= 1
    rng = np.random.default_rng(5)
    for _ in range(50):
        k = int(rng.integers(1, 5))
        b = [int(v) for v in rng.choice([1, 4, 8, 16, 32, 64, 128], k)]
        n, seg = int(rng.integers(1, 3000)), int(rng.choice([16, 64, 128]))
        lc, ic = float(rng.uniform(0, 1e-3)), float(rng.uniform(1e-6, 1e-4))
        own = oracle.fifo_hand_out(n, seg, b, lc, ic)
        segs = oracle.segments(n, seg)
        assert len(own) == len(segs) and all(0 <= o < k for o in own)
        cost = lambda w, a, e: len(oracle.batches(a, e, b[w])) * lc + (e - a) * ic      # noqa: E731
        load = [sum(cost(w, a, e) for o, (a, e) in zip(own, segs) if o == w) for w in range(k)]
        # the ideal split gives every worker the same finishing time T with sum_w T / cost_w(full segment) = #segments
        full = [cost(w, 0, seg) for w in range(k)]
        t_ideal = len(segs) / sum(1.0 / f for f in full)
        assert max(load) <= t_ideal + max(full) + 1e-12


def test_softmax_properties():
    z = RNG.standard_normal((5, 1000)) * 4
    p = oracle.softmax(z)
    np.testing.assert_allclose(p.sum(1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.softmax(z + 123.0), p, rtol=1e-12, atol=0)
    np.testing.assert_allclose(oracle.softmax(np.full((2, 10), 3.3)), 0.1, rtol=1e-15)
    np.testing.assert_allclose(p, scipy.special.softmax(z, axis=-1), rtol=1e-12, atol=0)
    p32 = oracle.softmax(z.astype(np.float32), dtype=np.float32)
    np.testing.assert_allclose(p32.sum(1), 1.0, atol=1e-6)
    big = oracle.softmax(np.array([[1000.0, 0.0, -1000.0]]))
    assert np.isfinite(big).all() and big[0, 0] == 1.0


def test_combination_rule_properties():
    ps = [oracle.softmax(RNG.standard_normal((9, 13)) * 3) for _ in range(4)]
    y = oracle.combine_mean(ps)
    np.testing.assert_allclose(y.sum(1), 1.0, atol=1e-14)
    np.testing.assert_allclose(y, np.mean(np.stack(ps), axis=0), rtol=1e-14)
    assert np.array_equal(oracle.combine_mean([ps[0]]), ps[0])                    # ensemble of one
    np.testing.assert_allclose(oracle.combine_mean([ps[1]] * 3), ps[1], rtol=1e-15)  # identical members
    np.testing.assert_allclose(oracle.combine_mean(ps[::-1]), y, rtol=1e-14)      # permutation


def test_message_accumulation_equals_direct_mean():
    """The accumulator loop over (s, m, P) triplets in a shuffled arrival order
    gives the plain mean (section 'The prediction accumulator')."""
    n, c, m, seg = 300, 7, 3, 128
    ps = [oracle.softmax(RNG.standard_normal((n, c))) for _ in range(m)]
    msgs = []
    for mi in range(m):
        for s, (a, b) in enumerate(oracle.segments(n, seg)):
            msgs.append((s, mi, ps[mi][a:b]))
    order = RNG.permutation(len(msgs))
    y = oracle.accumulate_messages([msgs[i] for i in order], n, c, m, seg)
    np.testing.assert_allclose(y, oracle.combine_mean(ps), rtol=1e-13)
    assert len(msgs) == m * 3


def test_top1_lowest_index_on_ties():
    assert list(oracle.top1(np.array([[0.2, 0.4, 0.4], [0.5, 0.5, 0.0]]))) == [1, 0]


def test_ensemble_of_one_equals_member_softmax():
    nets = N.config_members(1)
    blobs = [W.make_blob(n, synth.BASE_SEED, i) for i, n in enumerate(nets)]
    x = W.make_images(synth.BASE_SEED + 1000, 6, 32, 32)
    y, probs = oracle.ensemble_predict(nets, blobs, x, real="f64")
    np.testing.assert_allclose(y.sum(1), 1.0, atol=1e-12)
    y0, p0 = oracle.ensemble_predict(nets[:1], blobs[:1], x, real="f64")
    assert np.array_equal(y0, p0[0]) and np.array_equal(p0[0], probs[0])
    np.testing.assert_allclose(y, 0.5 * probs[0] + 0.5 * probs[1], rtol=1e-14)
    # a member's output does not depend on which other images share the call
    y_half, _ = oracle.ensemble_predict(nets, blobs, x[3:], real="f64")
    assert np.array_equal(y_half, y[3:])


def test_resize_pins():
    x = RNG.standard_normal((2, 10, 12, 3)).astype(np.float32)
    assert np.array_equal(oracle.resize_bilinear(x, 10, 12), x)
    const = np.full((1, 8, 8, 3), 1.75, np.float32)
    assert np.all(oracle.resize_bilinear(const, 11, 13) == 1.75)
    ramp = np.zeros((1, 16, 16, 1), np.float32)
    ramp[0, :, :, 0] = np.arange(16)[None, :] * 2.0 + 1.0
    out = oracle.resize_bilinear(ramp, 21, 21)[0, :, :, 0]
    src = (np.arange(21) + 0.5) * 16 / 21 - 0.5
    interior = (src >= 0) & (src <= 15)
    np.testing.assert_allclose(out[5, interior], src[interior] * 2.0 + 1.0, rtol=1e-6)
    big = oracle.resize_bilinear(x, 27, 31)
    ref = torch.nn.functional.interpolate(torch.from_numpy(x).double().permute(0, 3, 1, 2), size=(27, 31),
                                          mode="bilinear", align_corners=False).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(big, ref, rtol=0, atol=1e-6)
    up = oracle.resize_bilinear(W.make_images(3, 1, 224, 224), 299, 299)
    ref = torch.nn.functional.interpolate(torch.from_numpy(W.make_images(3, 1, 224, 224)).double().permute(0, 3, 1, 2),
                                          size=(299, 299), mode="bilinear", align_corners=False)
    np.testing.assert_allclose(up, ref.permute(0, 2, 3, 1).numpy(), rtol=0, atol=1e-6)


def test_throughput_arithmetic_from_paper():
    g = GOLD["throughput_example"]
    assert round(g["images"] / g["seconds"]) == g["img_per_sec"]
    assert g["overhead_seconds"] / g["seconds"] <= g["overhead_bound"]
    w = GOLD["weak_scaling"]
    assert round(100 * w["sixteen_gpus"] / (16 * w["one_gpu"])) == w["efficiency_percent"]


# --------------------------------------------------------------------------- other combination rules
def test_weighted_average_pins():
    """Weighted averaging (named in section "The prediction accumulator"): equal weights give the mean,
    a one-hot weight vector returns that member, rows sum to the sum of the weights, and the value
    equals a tensor contraction written independently."""
    rng = np.random.default_rng(5)
    probs = [oracle.softmax(rng.normal(size=(7, 11))) for _ in range(4)]
    w = np.array([0.1, 0.2, 0.3, 0.4])
    y = oracle.combine_weighted(probs, w)
    assert np.allclose(y, np.einsum("m,mic->ic", w, np.stack(probs)), atol=1e-15)
    assert np.allclose(y.sum(axis=1), 1.0, atol=1e-14)
    assert np.allclose(oracle.combine_weighted(probs, [0.25] * 4), oracle.combine_mean(probs), atol=1e-15)
    assert np.array_equal(oracle.combine_weighted(probs, [0, 0, 1, 0]), probs[2])
    assert np.allclose(oracle.combine_weighted(probs, 2 * w).sum(axis=1), 2.0)   # weights are used as given


def test_majority_vote_pins():
    """Majority voting: vote counts sum to M, a single member gives the one-hot of its arg-max, a
    hand-counted example, lowest index on exact ties, and agreement with a per-sample loop."""
    z = [np.array([[1.0, 3.0, 2.0], [5.0, 0.0, 5.0]]),
         np.array([[9.0, 1.0, 0.0], [0.0, 1.0, 2.0]]),
         np.array([[0.0, 2.0, 1.0], [0.0, 0.0, 1.0]])]
    y = oracle.combine_vote(z)
    # sample 0: votes 1, 0, 1 -> class 1 twice, class 0 once; sample 1: votes 0 (tie -> lowest), 2, 2
    assert np.allclose(y, np.array([[1, 2, 0], [1, 0, 2]]) / 3.0)
    assert np.allclose(y.sum(axis=1) * 3, 3.0)
    one = oracle.combine_vote([z[0]])
    assert np.array_equal(one, np.array([[0.0, 1.0, 0.0], [1.0, 0.0, 0.0]]))
    rng = np.random.default_rng(6)
    zs = [rng.normal(size=(20, 9)) for _ in range(5)]
    y = oracle.combine_vote(zs)
    for i in range(20):
        counts = np.zeros(9)
        for m in range(5):
            best = max(range(9), key=lambda c: (zs[m][i, c], -c))
            counts[best] += 1
        assert np.array_equal(y[i] * 5, counts)
    # softmax is monotone: voting on probabilities or on logits is the same
    assert np.array_equal(oracle.combine_vote([oracle.softmax(v) for v in zs]), y)
