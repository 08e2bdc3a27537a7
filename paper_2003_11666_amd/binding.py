"""ctypes binding of include/pb.h.  Argument marshalling only: every step of
the pipeline tick runs in the HIP library.  PyTorch provides device memory
(the arena, resident sample pools) and the stream."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

OP_KIND = {"linear": 0, "conv": 1, "gn": 2, "relu": 3, "maxpool": 4, "gap": 5, "add": 6, "ce": 7}

EXPORTS = ["pb_arena_bytes", "pb_init", "pb_init_static", "pb_static_arena_bytes", "pb_tick", "pb_run_resident", "pb_read_weights",
           "pb_read_velocity", "pb_loss_history", "pb_num_params", "pb_num_ticks",
           "pb_set_launch_mode", "pb_plan_summary", "pb_profile_begin", "pb_profile_end", "pb_update_standalone",
           "pb_scale_hyperparameters",
           "pb_sync", "pb_destroy", "pb_last_error"]


class PBError(RuntimeError):
    pass


class _Op(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "cin", "cout", "k", "stride", "pad", "groups",
                                         "has_bias", "skip_from_stage", "has_proj")]


class _Stage(C.Structure):
    _fields_ = [("n_ops", C.c_int32), ("ops", C.POINTER(_Op))]


class _Tuning(C.Structure):
    _fields_ = [("tile_target", C.c_int32), ("tile_target_bwd", C.c_int32), ("tile_budget_us", C.c_float),
                ("nt_stores", C.c_int32), ("one_launch", C.c_int32), ("tail_merge", C.c_int32), ("spin_limit", C.c_int32),
                ("dense_1x1", C.c_int32), ("gemm_lds_kb", C.c_int32)]


class _NetDesc(C.Structure):
    _fields_ = [("n_stages", C.c_int32), ("stages", C.POINTER(_Stage)),
                ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("n_classes", C.c_int32), ("mitigation", C.c_int32), ("bwd_weights", C.c_int32),
                ("act_dtype", C.c_int32), ("loss_capacity", C.c_int32), ("kernel_set", C.c_int32),
                ("device_arena", C.c_void_p), ("arena_bytes", C.c_size_t), ("stream", C.c_void_p),
                ("sc_scale", C.c_float), ("lwp_scale", C.c_float), ("lwp_form", C.c_int32),
                ("update_size", C.c_int32), ("tuning", C.POINTER(_Tuning))]


def lib_path():
    return os.path.join(_HERE, "libpb_hip.so")


def load_library():
    """Load libpb_hip.so; there is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime; it must be in the process first so that
    # the library binds to the same runtime instance that owns the tensors and
    # streams handed to it.
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise PBError(f"{path} is missing: build it with `python -m paper_2003_11666_amd.build`")
    lib = C.CDLL(path)
    fp, ip = C.POINTER(C.c_float), C.POINTER(C.c_int32)
    lib.pb_arena_bytes.restype = C.c_size_t
    lib.pb_arena_bytes.argtypes = [C.POINTER(_NetDesc), ip]
    lib.pb_init.restype = C.c_int
    lib.pb_init.argtypes = [C.POINTER(C.c_void_p), C.POINTER(_NetDesc), ip, C.c_float, C.c_float, C.c_uint64]
    lib.pb_init_static.restype = C.c_int
    lib.pb_init_static.argtypes = lib.pb_init.argtypes
    lib.pb_static_arena_bytes.restype = C.c_size_t
    lib.pb_static_arena_bytes.argtypes = []
    lib.pb_tick.restype = C.c_int
    lib.pb_tick.argtypes = [C.c_void_p, fp, C.c_int32]
    lib.pb_run_resident.restype = C.c_int
    lib.pb_run_resident.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64]
    for name in ("pb_read_weights", "pb_read_velocity", "pb_loss_history"):
        f = getattr(lib, name)
        f.restype = C.c_int64
        f.argtypes = [C.c_void_p, fp, C.c_int64]
    lib.pb_num_params.restype = C.c_int64
    lib.pb_num_params.argtypes = [C.c_void_p]
    lib.pb_num_ticks.restype = C.c_int64
    lib.pb_num_ticks.argtypes = [C.c_void_p]
    lib.pb_set_launch_mode.restype = C.c_int
    lib.pb_set_launch_mode.argtypes = [C.c_void_p, C.c_int32]
    lib.pb_profile_begin.restype = C.c_int
    lib.pb_profile_begin.argtypes = [C.c_void_p, C.c_int32]
    lib.pb_profile_end.restype = C.c_int
    lib.pb_profile_end.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.pb_update_standalone.restype = C.c_int
    lib.pb_update_standalone.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                         C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_void_p]
    lib.pb_plan_summary.restype = C.c_int64
    lib.pb_plan_summary.argtypes = [C.POINTER(_NetDesc), C.c_char_p, C.c_int64]
    lib.pb_scale_hyperparameters.restype = C.c_int
    lib.pb_scale_hyperparameters.argtypes = [C.c_float, C.c_float, C.c_int32, C.c_int32, fp, fp]
    lib.pb_sync.restype = C.c_int
    lib.pb_sync.argtypes = [C.c_void_p]
    lib.pb_destroy.restype = None
    lib.pb_destroy.argtypes = [C.c_void_p]
    lib.pb_last_error.restype = C.c_char_p
    lib.pb_last_error.argtypes = []
    _LIB = lib
    return lib


def _check(lib, rc):
    if rc < 0:
        raise PBError(f"pb error {rc}: {lib.pb_last_error().decode()}")
    return rc


def marshal_net(net, mitigation=3, bwd_weights=0, loss_capacity=0, kernel_set=0, sc_scale=1.0, lwp_scale=1.0, lwp_form="v",
                update_size=1, tuning=None):
    """dict descriptor (pb_workloads) -> pb_net_desc; returns (desc, keepalive)."""
    keep = []
    stages = (_Stage * len(net["stages"]))()
    for si, st in enumerate(net["stages"]):
        ops = (_Op * len(st))()
        for oi, o in enumerate(st):
            ops[oi] = _Op(OP_KIND[o["kind"]], o["cin"], o["cout"], o["k"], o["stride"], o["pad"],
                          o["groups"], o["bias"], o["skip_from"], o["proj"])
        keep.append(ops)
        stages[si] = _Stage(len(st), ops)
    keep.append(stages)
    d = _NetDesc()
    d.n_stages = len(net["stages"])
    d.stages = stages
    d.in_c, d.in_h, d.in_w = net["in_c"], net["in_h"], net["in_w"]
    d.n_classes = net["n_classes"]
    d.mitigation, d.bwd_weights = mitigation, bwd_weights
    d.sc_scale, d.lwp_scale = sc_scale, lwp_scale
    d.lwp_form = {"v": 0, "w": 1}[lwp_form]
    d.act_dtype = {"fp32": 0, "bf16": 1}[net.get("act_dtype", "fp32")]
    d.loss_capacity = loss_capacity
    d.kernel_set = kernel_set
    d.update_size = update_size
    if tuning:
        tn = _Tuning(**tuning)
        keep.append(tn)
        d.tuning = C.pointer(tn)
    return d, keep


def plan_summary(net, **kw):
    lib = load_library()
    desc, keep = marshal_net(net, **kw)
    n = lib.pb_plan_summary(C.byref(desc), None, 0)
    if n < 0:
        raise PBError(lib.pb_last_error().decode())
    buf = C.create_string_buffer(n)
    lib.pb_plan_summary(C.byref(desc), buf, n)
    return buf.value.decode()


class PBEngine:
    """pb_init / pb_tick / pb_run_resident / pb_read_weights / pb_loss_history."""

    def __init__(self, net, lr=None, momentum=None, seed=42, mitigation=3, delays=None,
                 bwd_weights=0, loss_capacity=0, torch_arena=True, kernel_set=0, sc_scale=1.0, lwp_scale=1.0, lwp_form="v",
                 static_arena=False, update_size=1, tuning=None):
        self.lib = load_library()
        self.net = net
        desc, self._keep = marshal_net(net, mitigation, bwd_weights, loss_capacity, kernel_set, sc_scale, lwp_scale, lwp_form,
                                       update_size, tuning)
        dl = None
        if delays is not None:
            dl = (C.c_int32 * len(delays))(*delays)
        self._arena = None
        if static_arena:
            import torch
            desc.stream = torch.cuda.current_stream().cuda_stream
        elif torch_arena:
            import torch
            need = self.lib.pb_arena_bytes(C.byref(desc), dl)
            if need == 0:
                raise PBError(f"pb_arena_bytes: {self.lib.pb_last_error().decode()}")
            self._arena = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
            ptr = (self._arena.data_ptr() + 255) // 256 * 256
            desc.device_arena = ptr
            desc.arena_bytes = need
            desc.stream = torch.cuda.current_stream().cuda_stream
        self.ctx = C.c_void_p()
        lr = net["lr"] if lr is None else lr
        momentum = net["momentum"] if momentum is None else momentum
        init = self.lib.pb_init_static if static_arena else self.lib.pb_init
        _check(self.lib, init(C.byref(self.ctx), C.byref(desc), dl, lr, momentum, seed))
        self.n_params = self.lib.pb_num_params(self.ctx)
        self._in_elems = net["in_c"] * net["in_h"] * net["in_w"]

    def tick(self, sample, label):
        x = np.ascontiguousarray(sample, dtype=np.float32).reshape(-1)
        assert x.size == self._in_elems
        _check(self.lib, self.lib.pb_tick(self.ctx, x.ctypes.data_as(C.POINTER(C.c_float)), int(label)))

    def run_resident(self, samples_dev, labels_dev, first_index, n_ticks):
        """samples_dev: float32 CUDA tensor [n_pool, ...]; labels_dev: int32 CUDA tensor [n_pool]."""
        assert samples_dev.is_cuda and labels_dev.is_cuda and samples_dev.is_contiguous()
        n_pool = labels_dev.numel()
        assert samples_dev.numel() == n_pool * self._in_elems
        _check(self.lib, self.lib.pb_run_resident(self.ctx, samples_dev.data_ptr(), labels_dev.data_ptr(),
                                                  n_pool, int(first_index), int(n_ticks)))

    def _read(self, fn, n):
        out = np.empty(n, dtype=np.float32)
        got = _check(self.lib, fn(self.ctx, out.ctypes.data_as(C.POINTER(C.c_float)), n))
        return out[:got]

    def read_weights(self):
        return self._read(self.lib.pb_read_weights, self.n_params)

    def read_velocity(self):
        return self._read(self.lib.pb_read_velocity, self.n_params)

    def loss_history(self):
        n = _check(self.lib, self.lib.pb_loss_history(self.ctx, None, 0))
        return self._read(self.lib.pb_loss_history, n) if n else np.empty(0, dtype=np.float32)

    @property
    def ticks(self):
        return self.lib.pb_num_ticks(self.ctx)

    def set_launch_mode(self, mode):
        _check(self.lib, self.lib.pb_set_launch_mode(self.ctx, mode))

    def profile_begin(self, max_events=1 << 16):
        _check(self.lib, self.lib.pb_profile_begin(self.ctx, max_events))

    def profile_end(self, which):
        n, ms = C.c_int64(), C.c_double()
        _check(self.lib, self.lib.pb_profile_end(self.ctx, which, C.byref(n), C.byref(ms)))
        return n.value, ms.value

    def sync(self):
        _check(self.lib, self.lib.pb_sync(self.ctx))

    def close(self):
        if self.ctx:
            self.lib.pb_destroy(self.ctx)
            self.ctx = C.c_void_p()
            self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def scale_hyperparameters(lr_ref, momentum_ref, n_ref, n=1):
    """(lr, momentum) for update size n from the reference values (pb_scale_hyperparameters)."""
    lib = load_library()
    lr, m = C.c_float(), C.c_float()
    _check(lib, lib.pb_scale_hyperparameters(lr_ref, momentum_ref, n_ref, n, C.byref(lr), C.byref(m)))
    return lr.value, m.value


def update_standalone(w, v, g, what, lr, m, a, b, lrT):
    """Fused update kernel over caller tensors (float32 CUDA, numel % 1024 == 0)."""
    import torch
    lib = load_library()
    _check(lib, lib.pb_update_standalone(w.data_ptr(), v.data_ptr(), g.data_ptr(),
                                         what.data_ptr() if what is not None else None, w.numel(),
                                         lr, m, a, b, lrT, torch.cuda.current_stream().cuda_stream))
