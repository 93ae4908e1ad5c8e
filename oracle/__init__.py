"""CPU oracle of the ensemble hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, direct implementations written from the paper's definitions and
the members' operation lists; imported by tests, the smoke check and the
benchmark's CPU-baseline leg only.  Shares no code with the GPU library.
"""
from .forward import forward_logits                      # noqa: F401
from .combine import (softmax, combine_mean, combine_weighted, combine_vote, segments, batches,   # noqa: F401
                      broadcast, accumulate_messages, top1, resize_bilinear, fifo_hand_out)
from . import planner                                      # noqa: F401


def ensemble_predict(nets, blobs, images, real="f32", store_bf16=False):
    """Combined class probabilities (n x C float64) of the ensemble on base-resolution
    `images`; each member is fed the images resized to its own resolution."""
    import numpy as np
    probs = []
    for net, blob in zip(nets, blobs):
        x = resize_bilinear(images, net.in_h, net.in_w)
        z = forward_logits(net, blob, x, real=real, store_bf16=store_bf16)
        dt = np.float32 if real == "f32" else np.float64
        probs.append(softmax(z.astype(dt), dtype=dt))
    return combine_mean(probs, dtype=np.float32 if real == "f32" else np.float64).astype(np.float64), probs
