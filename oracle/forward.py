"""Python face of the C forward-pass oracle (test infrastructure only)."""
import ctypes
import numpy as np
from . import build as _build

_FIELDS32 = ("kind", "src", "src_c0", "cin", "dst", "dst_c0", "cout", "kh", "kw", "sh", "sw",
             "pt", "pl", "act", "res", "res_c0", "pre", "r")
_FIELDS64 = ("off_w", "off_b", "off_bn", "off_pre", "off_w2", "off_b2")


class _Op(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in _FIELDS32] + [(f, ctypes.c_int64) for f in _FIELDS64]


class _Tensor(ctypes.Structure):
    _fields_ = [("h", ctypes.c_int32), ("w", ctypes.c_int32), ("c", ctypes.c_int32)]


_libs = {}


def _lib(real):
    if real not in _libs:
        _build.build()
        lib = ctypes.CDLL(_build.lib_path(real))
        lib.orc_forward.restype = ctypes.c_int
        lib.orc_forward.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        assert lib.orc_real_bytes() == (4 if real == "f32" else 8)
        _libs[real] = lib
    return _libs[real]


def forward_logits(net, blob, images, real="f32", store_bf16=False, dump_tensor=-1):
    """Logits (n x classes, float64 array) of member `net` with parameters `blob`
    on `images` (n x H x W x C fp32).  With dump_tensor >= 0 also returns that
    intermediate tensor of image 0."""
    lib = _lib(real)
    images = np.ascontiguousarray(images, dtype=np.float32)
    n = images.shape[0]
    assert images.shape[1:] == (net.in_h, net.in_w, net.in_c), images.shape
    blob = np.ascontiguousarray(blob, dtype=np.float32)
    assert blob.size == net.blob_size
    tens = (_Tensor * len(net.tensors))(*[_Tensor(*t) for t in net.tensors])
    ops = (_Op * len(net.ops))()
    for i, o in enumerate(net.ops):
        for f in _FIELDS32 + _FIELDS64:
            setattr(ops[i], f, int(o[f]))
    oh, ow, oc = net.tensors[net.out_tensor]
    out = np.zeros((n, oh * ow * oc), dtype=np.float64)
    dump = np.zeros(1, dtype=np.float64)
    if dump_tensor >= 0:
        dump = np.zeros(net.tensors[dump_tensor], dtype=np.float64)
    rc = lib.orc_forward(tens, len(net.tensors), ops, len(net.ops), blob.ctypes.data,
                         images.ctypes.data, n, net.out_tensor, out.ctypes.data,
                         int(store_bf16), dump_tensor, dump.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle forward failed (malformed description or out of memory)")
    return (out, dump) if dump_tensor >= 0 else out
