"""Oracle of the combination rule and the work partition (test infrastructure only).

Section "The prediction accumulator": the ensemble prediction is the average of
the members' prediction matrices, accumulated as Y[start(s):end(s)] += P / M
into a zeroed Y.  Section "The segment ids broadcaster": a request of nb_images
samples is cut into segments of N samples, start(s) = s*N,
end(s) = min((s+1)*N, nb_images).
"""
import numpy as np


def softmax(z, dtype=np.float64):
    """Row-wise softmax with the row maximum subtracted first."""
    z = np.asarray(z, dtype=dtype)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def combine_mean(member_probs, dtype=np.float64):
    """Y[i] = sum over members of P_m[i] / M, in member order."""
    m = len(member_probs)
    y = np.zeros_like(np.asarray(member_probs[0], dtype=dtype))
    for p in member_probs:
        y = y + np.asarray(p, dtype=dtype) / m
    return y


def combine_weighted(member_probs, weights, dtype=np.float64):
    """Weighted averaging, the first of the other combination rules the paper names (section "The
    prediction accumulator"): Y[i] = sum over members of w_m * P_m[i], in member order.  The weights
    are used as given; with w_m = 1/M this is combine_mean."""
    assert len(weights) == len(member_probs)
    y = np.zeros_like(np.asarray(member_probs[0], dtype=dtype))
    for p, w in zip(member_probs, weights):
        y = y + np.asarray(p, dtype=dtype) * dtype(w)
    return y


def combine_vote(member_logits, dtype=np.float64):
    """Majority voting, the second rule the paper names: every member votes for its arg-max class
    (lowest index on exact ties) and Y[i, c] = (number of members voting c for sample i) / M, so that
    a row still sums to one.  The winner of the vote is the arg-max of the row."""
    m = len(member_logits)
    z0 = np.asarray(member_logits[0])
    y = np.zeros(z0.shape, dtype=dtype)
    rows = np.arange(z0.shape[0])
    for z in member_logits:
        y[rows, np.argmax(np.asarray(z), axis=-1)] += 1.0
    return y / m


def segments(nb_images, seg):
    """[(start, end)] of every segment of a request of nb_images samples."""
    out = []
    s = 0
    while s * seg < nb_images:
        out.append((s * seg, min((s + 1) * seg, nb_images)))
        s += 1
    return out


def batches(start, end, b):
    """A segment cut into batches of the worker's batch size; the last one may be short."""
    return [(a, min(a + b, end)) for a in range(start, end, b)]


def broadcast(nb_images, seg, n_models):
    """Messages the broadcaster emits: every segment id once into each model's queue."""
    ids = list(range(len(segments(nb_images, seg))))
    return {m: list(ids) for m in range(n_models)}


def fifo_hand_out(nb_images, seg, worker_batches, launch_cost, image_cost):
    """Which worker of one DNN predicts which segment when all of them take segment ids from the same
    FIFO queue (section "Data-parallelism"), in a model of time where a worker with batch size b
    needs ceil(L / b) * launch_cost + L * image_cost for a segment of L samples.  Event simulation: a
    heap of (time the worker becomes idle, worker); the idle worker with the earliest time (lowest
    index among equals) pops the next id.  Returns the owner of every segment."""
    import heapq
    idle = [(0.0, k) for k in range(len(worker_batches))]
    heapq.heapify(idle)
    owners = []
    for (a, b) in segments(nb_images, seg):
        t, k = heapq.heappop(idle)
        duration = len(batches(a, b, worker_batches[k])) * launch_cost + (b - a) * image_cost
        heapq.heappush(idle, (t + duration, k))
        owners.append(k)
    return owners


def accumulate_messages(messages, nb_images, n_classes, n_models, seg, dtype=np.float64):
    """The accumulator as the paper runs it: a zeroed Y updated by each arriving
    triplet (s, m, P) in whatever order the messages come."""
    y = np.zeros((nb_images, n_classes), dtype=dtype)
    for (s, _m, p) in messages:
        a, b = s * seg, min((s + 1) * seg, nb_images)
        y[a:b] += np.asarray(p, dtype=dtype) / n_models
    return y


def top1(y):
    """Arg-max per row, lowest index on exact ties."""
    return np.argmax(y, axis=-1)


def resize_bilinear(images, out_h, out_w):
    """Bilinear resize, half-pixel centres, edge clamp, no antialiasing (fp64 maths)."""
    x = np.asarray(images, dtype=np.float64)
    n, h, w, c = x.shape
    if (h, w) == (out_h, out_w):
        return x.astype(np.float32)

    def axis(n_in, n_out):
        src = (np.arange(n_out) + 0.5) * (n_in / n_out) - 0.5
        src = np.clip(src, 0.0, n_in - 1.0)
        i0 = np.floor(src).astype(np.int64)
        i1 = np.minimum(i0 + 1, n_in - 1)
        return i0, i1, src - i0

    h0, h1, fh = axis(h, out_h)
    w0, w1, fw = axis(w, out_w)
    top = x[:, h0][:, :, w0] * (1 - fw)[None, None, :, None] + x[:, h0][:, :, w1] * fw[None, None, :, None]
    bot = x[:, h1][:, :, w0] * (1 - fw)[None, None, :, None] + x[:, h1][:, :, w1] * fw[None, None, :, None]
    out = top * (1 - fh)[None, :, None, None] + bot * fh[None, :, None, None]
    return out.astype(np.float32)
