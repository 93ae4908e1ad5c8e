"""Seeded parameter blobs and input images for the synthetic workloads.

Parameter rules (per parameter tensor t of member m, stream key(seed, m, t, kind)):
  conv / FC / SE weights : N(0, std^2), std = sqrt(gain / fan_in) (He-normal, gain 2;
                           FC heads use gain 1), layout [kh][kw][cin][cout]
  biases                 : N(0, 0.1^2)  (non-zero so that the bias path is exercised)
  batch-norm             : gamma constant (1, or the residual-branch constant),
                           beta 0, mean N(0, 0.1^2), variance U(0.5, 1.5)
Images: N(0, 1) per element, NHWC, stream key(seed, image index, 0, KIND_IMAGE).
"""
import numpy as np
from . import rng


def make_blob(net, seed, member):
    blob = np.zeros(net.blob_size, dtype=np.float32)
    for p in net.params:
        o, s, t = p["offset"], p["size"], p["index"]
        if p["role"] == "conv_w":
            k = rng.stream_key(seed, member, t, rng.KIND_WEIGHT)
            blob[o:o + s] = (rng.normal(k, s) * p["std"]).astype(np.float32)
        elif p["role"] == "bias":
            k = rng.stream_key(seed, member, t, rng.KIND_BIAS)
            blob[o:o + s] = (rng.normal(k, s) * 0.1).astype(np.float32)
        elif p["role"] == "bn":
            c = p["channels"]
            blob[o:o + c] = p["gamma"]
            blob[o + c:o + 2 * c] = 0.0
            k = rng.stream_key(seed, member, t, rng.KIND_BN_MEAN)
            blob[o + 2 * c:o + 3 * c] = (rng.normal(k, c) * 0.1).astype(np.float32)
            k = rng.stream_key(seed, member, t, rng.KIND_BN_VAR)
            blob[o + 3 * c:o + 4 * c] = rng.uniform_range(k, c, 0.5, 1.5).astype(np.float32)
        else:
            raise ValueError(p["role"])
    return blob


def make_images(seed, n, h, w, c=3, first=0, varied=False):
    """N(0, 1) images.  varied=True additionally gives every image its own contrast
    (uniform in [0.25, 1.75]) and per-channel offset (N(0, 1)), so that random-weight members,
    which average white noise away, answer differently from image to image."""
    out = np.empty((n, h, w, c), dtype=np.float32)
    per = h * w * c
    for i in range(n):
        k = rng.stream_key(seed, first + i, 0, rng.KIND_IMAGE)
        img = rng.normal(k, per).reshape(h, w, c)
        if varied:
            k2 = rng.stream_key(seed, first + i, 1, rng.KIND_IMAGE)
            gain = rng.uniform_range(k2, 1, 0.25, 1.75)[0]
            off = rng.normal(k2, c, start=1)
            img = img * gain + off.reshape(1, 1, c)
        out[i] = img.astype(np.float32)
    return out


def round_bf16(x):
    """Round fp32 values to the nearest bf16-representable value (ties to even)."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def quantise_weights_bf16(net, blob):
    """Copy of `blob` with the conv / FC / SE weight tensors rounded to bf16
    (biases and batch-norm statistics stay fp32)."""
    out = blob.copy()
    for p in net.params:
        if p["role"] == "conv_w":
            o, s = p["offset"], p["size"]
            out[o:o + s] = round_bf16(out[o:o + s])
    return out
