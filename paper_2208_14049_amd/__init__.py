"""Python binding of the MI355X ensemble-inference library (argument marshalling only).

Every step of the hot path runs inside libens_mi355x.so; this module converts member
descriptions and numpy / torch buffers to the C structures of include/ens.h and back.
It fails loudly when the library has not been built: there is no CPU fallback.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libens_mi355x.so")

ENS_OK, ENS_E_INVALID, ENS_E_NOMEM, ENS_E_NOFIT, ENS_E_HIP, ENS_E_NODEVICE, ENS_E_UNSUPPORTED, ENS_E_TOOBIG = 0, -1, -2, -3, -4, -5, -6, -7
ENS_FP32, ENS_BF16 = 0, 1
ENS_MAX_SLOTS, ENS_MAX_MEMBERS, ENS_MAX_DOMAIN = 16, 64, 16

_OP32 = ("kind", "src", "src_c0", "cin", "dst", "dst_c0", "cout", "kh", "kw", "sh", "sw",
         "pt", "pl", "act", "res", "res_c0", "pre", "r")
_OP64 = ("off_w", "off_b", "off_bn", "off_pre", "off_w2", "off_b2")


class EnsTensor(ctypes.Structure):
    _fields_ = [("h", ctypes.c_int32), ("w", ctypes.c_int32), ("c", ctypes.c_int32)]


class EnsOp(ctypes.Structure):
    _fields_ = [(f, ctypes.c_int32) for f in _OP32] + [(f, ctypes.c_int64) for f in _OP64]


class EnsParam(ctypes.Structure):
    _fields_ = [("role", ctypes.c_int32), ("channels", ctypes.c_int32), ("offset", ctypes.c_int64),
                ("size", ctypes.c_int64), ("scale", ctypes.c_double)]


class EnsMemberSpec(ctypes.Structure):
    _fields_ = [("tensors", ctypes.POINTER(EnsTensor)), ("n_tensors", ctypes.c_int32),
                ("ops", ctypes.POINTER(EnsOp)), ("n_ops", ctypes.c_int32),
                ("out_tensor", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("params", ctypes.POINTER(ctypes.c_float)), ("n_params", ctypes.c_int64),
                ("param_specs", ctypes.POINTER(EnsParam)), ("n_param_specs", ctypes.c_int32)]


class EnsAlloc(ctypes.Structure):
    _fields_ = [("rows", ctypes.c_int32), ("cols", ctypes.c_int32),
                ("batch", (ctypes.c_int32 * ENS_MAX_MEMBERS) * ENS_MAX_SLOTS),
                ("bytes", ctypes.c_int64), ("score", ctypes.c_double), ("n_bench", ctypes.c_int32)]

    def matrix(self):
        return [[self.batch[r][c] for c in range(self.cols)] for r in range(self.rows)]


class EnsPlanOpts(ctypes.Structure):
    _fields_ = [("n_domain", ctypes.c_int32), ("domain", ctypes.c_int32 * ENS_MAX_DOMAIN),
                ("default_batch", ctypes.c_int32), ("segment_size", ctypes.c_int32),
                ("max_neighs", ctypes.c_int32), ("max_iter", ctypes.c_int32), ("slots", ctypes.c_int32),
                ("strategy", ctypes.c_int32), ("seed", ctypes.c_uint64), ("n_calib", ctypes.c_int64),
                ("repeats", ctypes.c_int32), ("verbose", ctypes.c_int32)]


class EnsPlanProblem(ctypes.Structure):
    _fields_ = [("n_models", ctypes.c_int32), ("n_rows", ctypes.c_int32), ("n_pools", ctypes.c_int32),
                ("n_domain", ctypes.c_int32), ("domain", ctypes.POINTER(ctypes.c_int32)),
                ("default_batch", ctypes.c_int32), ("weight_bytes", ctypes.POINTER(ctypes.c_int64)),
                ("arena_bytes", ctypes.POINTER(ctypes.c_int64)), ("row_pool", ctypes.POINTER(ctypes.c_int32)),
                ("row_is_gpu", ctypes.POINTER(ctypes.c_int32)), ("pool_cap", ctypes.POINTER(ctypes.c_int64)),
                ("max_iter", ctypes.c_int32), ("max_neighs", ctypes.c_int32), ("seed", ctypes.c_uint64)]


BENCH_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p)
BENCH_SINGLE_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p)

EXPORTS = ("ens_load", "ens_free", "ens_set_io", "ens_plan", "ens_set_alloc", "ens_bench", "ens_predict",
           "ens_predict_static", "ens_static_scratch_bytes",
           "ens_member_logits", "ens_debug_tensor", "ens_debug_keep_tensors", "ens_classes", "ens_n_members", "ens_member_bytes",
           "ens_spec_bytes", "ens_set_profiling", "ens_debug_one_stream", "ens_profile_get", "ens_last_ms", "ens_set_combination", "ens_debug_fake_predictor",
           "ens_planner_fit_mem", "ens_planner_wfd", "ens_planner_neighbors", "ens_planner_greedy",
           "ens_planner_bbs", "ens_partition", "ens_hand_out", "ens_strerror", "ens_version")

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it first (python -m paper_2208_14049_amd.build); "
                               "there is no fallback path" % LIB_PATH)
        # PyTorch owns the process's HIP runtime (its device tensors are what callers hand in):
        # import it first so that the library binds to the same runtime instead of a second copy.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_double
        P = ctypes.POINTER
        L.ens_load.argtypes = [P(EnsMemberSpec), i32, u64, P(vp)]
        L.ens_free.argtypes = [vp]
        L.ens_free.restype = None
        L.ens_set_io.argtypes = [vp, i32, i32, i32, i32]
        L.ens_plan.argtypes = [vp, u64, P(EnsPlanOpts), P(EnsAlloc)]
        L.ens_set_alloc.argtypes = [vp, P(EnsAlloc), i32]
        L.ens_bench.argtypes = [vp, P(EnsAlloc), i32, i64, i32, P(dbl)]
        L.ens_predict.argtypes = [vp, vp, i64, vp]
        L.ens_predict_static.argtypes = [vp, vp, i64, vp]
        L.ens_member_logits.argtypes = [vp, i32, i64, vp]
        L.ens_debug_tensor.argtypes = [vp, i32, i32, i32, vp]
        L.ens_debug_keep_tensors.argtypes = [vp, i32]
        L.ens_classes.argtypes = [vp]
        L.ens_n_members.argtypes = [vp]
        L.ens_member_bytes.argtypes = [vp, i32, i32, P(i64), P(i64)]
        L.ens_spec_bytes.argtypes = [P(EnsMemberSpec), i32, P(i64), P(i64)]
        L.ens_set_profiling.argtypes = [vp, i32]
        L.ens_debug_one_stream.argtypes = [vp, i32]
        L.ens_set_combination.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_float)]
        L.ens_debug_fake_predictor.argtypes = [vp, i32]
        L.ens_profile_get.argtypes = [vp, i32, ctypes.c_char_p, i32, P(dbl), P(i64), P(dbl), P(dbl)]
        L.ens_last_ms.argtypes = [vp]
        L.ens_last_ms.restype = dbl
        L.ens_planner_fit_mem.argtypes = [P(EnsPlanProblem), P(i32)]
        L.ens_planner_wfd.argtypes = [P(EnsPlanProblem), P(i32)]
        L.ens_planner_neighbors.argtypes = [P(EnsPlanProblem), P(i32), P(i32), i32, P(i32)]
        L.ens_planner_greedy.argtypes = [P(EnsPlanProblem), P(i32), BENCH_FN, vp, P(dbl), P(i32)]
        L.ens_planner_bbs.argtypes = [P(EnsPlanProblem), BENCH_SINGLE_FN, vp, P(i32), P(i32)]
        L.ens_partition.argtypes = [i64, i32, i32, P(i64), P(i64), i32, P(i32)]
        L.ens_hand_out.argtypes = [i64, i32, P(i32), i32, dbl, dbl, P(i32), i32, P(i32)]
        L.ens_strerror.argtypes = [ctypes.c_int]
        L.ens_strerror.restype = ctypes.c_char_p
        L.ens_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


class EnsError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        RuntimeError.__init__(self, "%s: %s (%d)" % (where, lib().ens_strerror(status).decode(), status))


def _check(status, where):
    if status != ENS_OK:
        raise EnsError(status, where)


_ROLE = {"conv_w": 1, "bias": 2, "bn": 3}


def member_spec(net, params=None):
    """C description of one member.  `net` exposes tensors, ops (dicts), out_tensor, dtype,
    blob_size and params (as synth.nets.Net does).  Returns (spec, keep-alive objects)."""
    tens = (EnsTensor * len(net.tensors))(*[EnsTensor(*t) for t in net.tensors])
    ops = (EnsOp * len(net.ops))()
    for i, o in enumerate(net.ops):
        for f in _OP32 + _OP64:
            setattr(ops[i], f, int(o[f]))
    pspecs = (EnsParam * len(net.params))()
    for i, p in enumerate(net.params):
        pspecs[i].role = _ROLE[p["role"]]
        pspecs[i].channels = int(p.get("channels", 0))
        pspecs[i].offset = int(p["offset"])
        pspecs[i].size = int(p["size"])
        pspecs[i].scale = float(p.get("std", p.get("gamma", 0.0)))
    spec = EnsMemberSpec()
    spec.tensors, spec.n_tensors = tens, len(net.tensors)
    spec.ops, spec.n_ops = ops, len(net.ops)
    spec.out_tensor = net.out_tensor
    spec.dtype = ENS_BF16 if net.dtype == "bf16" else ENS_FP32
    keep = [tens, ops, pspecs]
    if params is not None:
        arr = np.ascontiguousarray(params, dtype=np.float32)
        assert arr.size == net.blob_size
        spec.params = arr.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
        keep.append(arr)
    else:
        spec.params = None
    spec.n_params = net.blob_size
    spec.param_specs, spec.n_param_specs = pspecs, len(net.params)
    return spec, keep


def _ptr(buf):
    """Raw address of a numpy array (host) or a torch tensor (host or device)."""
    if isinstance(buf, np.ndarray):
        return buf.ctypes.data
    return buf.data_ptr()


def _is_device(buf):
    return (not isinstance(buf, np.ndarray)) and getattr(buf, "is_cuda", False)


def _sync_producer(tensor):
    """The library runs on its own streams: what torch's current stream still has to write into a
    device tensor must have landed before the library reads it."""
    import torch
    torch.cuda.current_stream(tensor.device).synchronize()


def make_alloc(matrix):
    a = EnsAlloc()
    a.rows, a.cols = len(matrix), len(matrix[0])
    for r, row in enumerate(matrix):
        for c, v in enumerate(row):
            a.batch[r][c] = int(v)
    return a


class Ensemble:
    """An ensemble resident on the GPU.  Thin wrapper over the ens_* entry points."""

    def __init__(self, nets, params=None, seed=0):
        self._keep = []
        specs = (EnsMemberSpec * len(nets))()
        for i, net in enumerate(nets):
            sp, keep = member_spec(net, None if params is None else params[i])
            specs[i] = sp
            self._keep.append(keep)
        self._h = ctypes.c_void_p()
        _check(lib().ens_load(specs, len(nets), seed, ctypes.byref(self._h)), "ens_load")
        self.n_members = len(nets)
        self.classes = lib().ens_classes(self._h)
        self.base_hw = (nets[0].in_h, nets[0].in_w)
        self._io = None

    def close(self):
        if self._h:
            lib().ens_free(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_base_size(self, h, w):
        self.base_hw = (h, w)
        self._io = None

    def _set_io(self, images_dev, probs_dev):
        key = (self.base_hw, images_dev, probs_dev)
        if key != self._io:
            _check(lib().ens_set_io(self._h, self.base_hw[0], self.base_hw[1], int(images_dev), int(probs_dev)), "ens_set_io")
            self._io = key

    def ens_set_alloc(self, matrix, segment_size=128):
        a = make_alloc(matrix)
        _check(lib().ens_set_alloc(self._h, ctypes.byref(a), segment_size), "ens_set_alloc")

    def ens_plan(self, mem_budget_bytes=0, **opts):
        o = EnsPlanOpts()
        dom = opts.pop("domain", None)
        if dom:
            o.n_domain = len(dom)
            for i, v in enumerate(dom):
                o.domain[i] = v
        for k, v in opts.items():
            setattr(o, k, v)
        self._set_io(True, True)
        out = EnsAlloc()
        _check(lib().ens_plan(self._h, int(mem_budget_bytes), ctypes.byref(o), ctypes.byref(out)), "ens_plan")
        return out

    def ens_bench(self, matrix, n_calib=1024, segment_size=128, repeats=3):
        a = make_alloc(matrix)
        ips = ctypes.c_double(0.0)
        _check(lib().ens_bench(self._h, ctypes.byref(a), segment_size, n_calib, repeats, ctypes.byref(ips)), "ens_bench")
        return ips.value

    def ens_predict(self, images, out=None):
        """images: n x H x W x 3 fp32, numpy (host) or torch (host or device) -> n x classes fp32."""
        n = int(images.shape[0])
        assert tuple(images.shape[1:]) == (self.base_hw[0], self.base_hw[1], 3), images.shape
        dev_in = _is_device(images)
        if isinstance(images, np.ndarray):
            images = np.ascontiguousarray(images, dtype=np.float32)
        else:
            assert images.is_contiguous() and str(images.dtype) == "torch.float32"
        if out is None:
            if dev_in:
                import torch
                out = torch.empty((n, self.classes), dtype=torch.float32, device=images.device)
            else:
                out = np.empty((n, self.classes), dtype=np.float32)
        self._set_io(dev_in, _is_device(out))
        if dev_in:
            _sync_producer(images)
        _check(lib().ens_predict(self._h, _ptr(images), n, _ptr(out)), "ens_predict")
        return out

    def ens_predict_static(self, images, out):
        """ens_predict without device allocations: images and out are torch device tensors."""
        n = int(images.shape[0])
        assert tuple(images.shape[1:]) == (self.base_hw[0], self.base_hw[1], 3), images.shape
        assert _is_device(images) and _is_device(out), "device tensors only"
        assert images.is_contiguous() and str(images.dtype) == "torch.float32"
        assert out.is_contiguous() and str(out.dtype) == "torch.float32" and tuple(out.shape) == (n, self.classes)
        self._set_io(True, True)
        _sync_producer(images)
        _check(lib().ens_predict_static(self._h, _ptr(images), n, _ptr(out)), "ens_predict_static")
        return out

    def ens_member_logits(self, member, n):
        out = np.empty((n, self.classes), dtype=np.float32)
        _check(lib().ens_member_logits(self._h, member, n, out.ctypes.data), "ens_member_logits")
        return out

    def ens_debug_tensor(self, member, tensor, shape_hwc, n_images):
        out = np.empty((n_images,) + tuple(shape_hwc), dtype=np.float32)
        _check(lib().ens_debug_tensor(self._h, member, tensor, n_images, out.ctypes.data), "ens_debug_tensor")
        return out

    def ens_debug_keep_tensors(self, on=True):
        _check(lib().ens_debug_keep_tensors(self._h, int(on)), "ens_debug_keep_tensors")

    def ens_member_bytes(self, member, batch):
        w, a = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().ens_member_bytes(self._h, member, batch, ctypes.byref(w), ctypes.byref(a)), "ens_member_bytes")
        return w.value, a.value

    def ens_set_combination(self, rule, weights=None):
        """rule: "mean", "weighted" (weights: one float per member) or "vote"."""
        code = {"mean": 0, "weighted": 1, "vote": 2}[rule]
        w = None
        if weights is not None:
            w = (ctypes.c_float * len(weights))(*[float(v) for v in weights])
        _check(lib().ens_set_combination(self._h, code, w), "ens_set_combination")

    def ens_debug_fake_predictor(self, on):
        _check(lib().ens_debug_fake_predictor(self._h, int(on)), "ens_debug_fake_predictor")

    def ens_set_profiling(self, on):
        _check(lib().ens_set_profiling(self._h, int(on)), "ens_set_profiling")

    def ens_debug_one_stream(self, on):
        _check(lib().ens_debug_one_stream(self._h, int(on)), "ens_debug_one_stream")

    def ens_profile(self):
        """[{name, ms, launches, flop, bytes}] of the last profiled call."""
        out = []
        i = 0
        while True:
            name = ctypes.create_string_buffer(128)
            ms, fl, by, ln = ctypes.c_double(), ctypes.c_double(), ctypes.c_double(), ctypes.c_int64()
            rc = lib().ens_profile_get(self._h, i, name, 128, ctypes.byref(ms), ctypes.byref(ln), ctypes.byref(fl), ctypes.byref(by))
            if rc != ENS_OK:
                break
            out.append(dict(name=name.value.decode(), ms=ms.value, launches=ln.value, flop=fl.value, bytes=by.value))
            i += 1
        return out

    def ens_last_ms(self):
        return lib().ens_last_ms(self._h)


def ens_spec_bytes(net, batch):
    spec, keep = member_spec(net, None)
    w, a = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().ens_spec_bytes(ctypes.byref(spec), batch, ctypes.byref(w), ctypes.byref(a)), "ens_spec_bytes")
    return w.value, a.value


def ens_partition(nb_images, segment_size, batch):
    n = ctypes.c_int32()
    _check(lib().ens_partition(nb_images, segment_size, batch, None, None, 0, ctypes.byref(n)), "ens_partition")
    st = (ctypes.c_int64 * max(1, n.value))()
    en = (ctypes.c_int64 * max(1, n.value))()
    _check(lib().ens_partition(nb_images, segment_size, batch, st, en, n.value, ctypes.byref(n)), "ens_partition")
    return [(st[i], en[i]) for i in range(n.value)]


def ens_hand_out(nb_images, segment_size, batches, launch_cost, image_cost):
    """Owner (worker index) of every segment of one member's request."""
    b = (ctypes.c_int32 * len(batches))(*[int(v) for v in batches])
    n = ctypes.c_int32()
    _check(lib().ens_hand_out(nb_images, segment_size, b, len(batches), launch_cost, image_cost, None, 0, ctypes.byref(n)), "ens_hand_out")
    out = (ctypes.c_int32 * max(1, n.value))()
    _check(lib().ens_hand_out(nb_images, segment_size, b, len(batches), launch_cost, image_cost, out, n.value, ctypes.byref(n)), "ens_hand_out")
    return [out[i] for i in range(n.value)]


class PlanProblem:
    """Marshals the host-only planner's problem description."""

    def __init__(self, weight_bytes, arena_bytes, domain, default_batch, row_pool, row_is_gpu, pool_cap,
                 max_iter=10, max_neighs=100, seed=0):
        self.n_models, self.n_rows = len(weight_bytes), len(row_pool)
        self._dom = (ctypes.c_int32 * len(domain))(*domain)
        self._w = (ctypes.c_int64 * self.n_models)(*weight_bytes)
        flat = [int(v) for row in arena_bytes for v in row]
        self._a = (ctypes.c_int64 * len(flat))(*flat)
        self._rp = (ctypes.c_int32 * self.n_rows)(*row_pool)
        self._rg = (ctypes.c_int32 * self.n_rows)(*[int(bool(g)) for g in row_is_gpu])
        self._cap = (ctypes.c_int64 * len(pool_cap))(*pool_cap)
        p = EnsPlanProblem()
        p.n_models, p.n_rows, p.n_pools, p.n_domain = self.n_models, self.n_rows, len(pool_cap), len(domain)
        p.domain, p.default_batch = self._dom, default_batch
        p.weight_bytes, p.arena_bytes = self._w, self._a
        p.row_pool, p.row_is_gpu, p.pool_cap = self._rp, self._rg, self._cap
        p.max_iter, p.max_neighs, p.seed = max_iter, max_neighs, seed
        self.c = p

    def _flat(self, matrix):
        return (ctypes.c_int32 * (self.n_rows * self.n_models))(*[int(v) for row in matrix for v in row])

    def _unflat(self, arr, off=0):
        M = self.n_models
        return [[arr[off + r * M + c] for c in range(M)] for r in range(self.n_rows)]

    def fit_mem(self, matrix):
        rc = lib().ens_planner_fit_mem(ctypes.byref(self.c), self._flat(matrix))
        if rc < 0:
            raise EnsError(rc, "ens_planner_fit_mem")
        return bool(rc)

    def wfd(self):
        out = (ctypes.c_int32 * (self.n_rows * self.n_models))()
        _check(lib().ens_planner_wfd(ctypes.byref(self.c), out), "ens_planner_wfd")
        return self._unflat(out)

    def neighbors(self, matrix):
        n = ctypes.c_int32()
        flat = self._flat(matrix)
        _check(lib().ens_planner_neighbors(ctypes.byref(self.c), flat, None, 0, ctypes.byref(n)), "ens_planner_neighbors")
        cells = self.n_rows * self.n_models
        out = (ctypes.c_int32 * max(1, n.value * cells))()
        _check(lib().ens_planner_neighbors(ctypes.byref(self.c), flat, out, n.value, ctypes.byref(n)), "ens_planner_neighbors")
        return [self._unflat(out, i * cells) for i in range(n.value)]

    def greedy(self, matrix, bench):
        flat = self._flat(matrix)
        cells = self.n_rows * self.n_models

        def cb(ptr, _user):
            return float(bench(self._unflat([ptr[i] for i in range(cells)])))

        score, nb = ctypes.c_double(), ctypes.c_int32()
        _check(lib().ens_planner_greedy(ctypes.byref(self.c), flat, BENCH_FN(cb), None, ctypes.byref(score), ctypes.byref(nb)),
               "ens_planner_greedy")
        return self._unflat(flat), score.value, nb.value

    def bbs(self, bench_single):
        out = (ctypes.c_int32 * self.n_models)()
        nb = ctypes.c_int32()
        cb = BENCH_SINGLE_FN(lambda m, b, _u: float(bench_single(m, b)))
        _check(lib().ens_planner_bbs(ctypes.byref(self.c), cb, None, out, ctypes.byref(nb)), "ens_planner_bbs")
        return list(out), nb.value
