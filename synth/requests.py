"""Seeded requests for the full-size parity cases of workload configurations 2-5.

Inputs only: member descriptions, their parameter blobs (convolution / FC weights rounded to
bf16 once, so that both sides are fed the same values) and the request images, also rounded to
bf16.  A request mixes the workload's own distribution with images that make random-weight
members answer differently from image to image: the first eighth is plain N(0, 1), the rest has
per-image contrast and per-channel offsets (`weights.make_images(..., varied=True)`).
"""
from . import nets as N
from . import weights as W

BASE_SEED = 220814049

# request sizes of the full-size parity cases (the heavy 12-member ensemble takes half the images)
FULL_SIZE_N = {2: 256, 3: 256, 4: 128, 5: 256}


def full_size_case(cfg, n=None):
    """(nets, blobs, images) of configuration `cfg` at its full input size; images n x 224 x 224 x 3."""
    nets = N.config_members(cfg)
    n = FULL_SIZE_N[cfg] if n is None else n
    size = N.BASE_SIZE[cfg]
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, BASE_SEED, i)) for i, net in enumerate(nets)]
    plain = n // 8
    imgs = W.make_images(BASE_SEED + 1000, n, size, size)
    imgs[plain:] = W.make_images(BASE_SEED + 1000, n - plain, size, size, first=plain, varied=True)
    return nets, blobs, W.round_bf16(imgs)
