"""The allocation-free entry point (ens_predict_static) against ens_predict.

Both run the same kernels; the only difference is where the members' logits of the request live
(library allocations vs the fixed device array), so the outputs are compared bit for bit, on
two calls in a row, the second with a smaller request.
"""
import numpy as np
import pytest

import synth
from synth import nets as N
from synth import weights as W

pytestmark = pytest.mark.gpu


def test_static_entry_point_matches_ens_predict():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_2208_14049_amd as ens
    L = ens.lib()
    assert L.ens_static_scratch_bytes() == 32 << 20
    nets = [N.resnet18(size=64, classes=100), N.efficientnet(0, size=64, classes=100), N.densenet121(size=64, classes=100)]
    blobs = [W.quantise_weights_bf16(net, W.make_blob(net, synth.BASE_SEED + 3, i)) for i, net in enumerate(nets)]
    imgs = torch.from_numpy(W.round_bf16(W.make_images(synth.BASE_SEED + 1000, 200, 64, 64, varied=True))).cuda()
    E = ens.Ensemble(nets, blobs)
    E.ens_set_alloc([[16, 8, 32], [8, 0, 0]], 64)                # two workers for member 0; segments of 64
    sizes = (200, 77)                                            # ragged last segment and batch; then a smaller request
    want = []
    for n in sizes:
        want.append(E.ens_predict(imgs[:n].contiguous()).cpu().numpy())
    z_want = E.ens_member_logits(1, sizes[-1])
    for n, ref in zip(sizes, want):
        out = torch.full((n, E.classes), -1.0, device="cuda")
        E.ens_predict_static(imgs[:n].contiguous(), out)
        got = out.cpu().numpy()
        assert np.isfinite(got).all() and np.abs(got.sum(1) - 1.0).max() <= 1e-4
        assert np.array_equal(got, ref), (n, float(np.abs(got - ref).max()))
    assert np.array_equal(E.ens_member_logits(1, sizes[-1]), z_want)     # read from the fixed array
    # back on the library's own buffers, and once more on the fixed array
    assert np.array_equal(E.ens_predict(imgs[:77].contiguous()).cpu().numpy(), want[1])
    out = torch.empty((77, E.classes), device="cuda")
    E.ens_predict_static(imgs[:77].contiguous(), out)
    assert np.array_equal(out.cpu().numpy(), want[1])
    # beyond the fixed array: refused before anything runs (3 members x 100 classes: 27 959 rows at most)
    cap = ((32 << 20) - 4096) // (3 * 100 * 4)
    big = torch.zeros((1, 64, 64, 3), device="cuda")
    rc = L.ens_predict_static(E._h, big.data_ptr(), cap + 1, out.data_ptr())
    assert rc == ens.ENS_E_TOOBIG and b"static scratch" in L.ens_strerror(rc)
    E.ens_set_profiling(1)
    with pytest.raises(ens.EnsError):
        E.ens_predict_static(imgs[:77].contiguous(), out)
    E.ens_set_profiling(0)
    E.close()
    # without an installed allocation the call is refused (installing one allocates the arenas)
    E2 = ens.Ensemble(nets[:1], blobs[:1])
    with pytest.raises(ens.EnsError):
        E2.ens_predict_static(imgs[:8].contiguous(), torch.empty((8, E2.classes), device="cuda"))
    E2.close()
