"""Thin ctypes binding of the SelSync C ABI (``include/selsync.h``).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libselsync.so``.  PyTorch is used for device memory (``tensor.data_ptr()``) and for
the current HIP stream, nothing else.  There is no CPU fallback: if the library has
not been built, importing this module raises.

The raw C entry points are available under their C names (``selsync_step`` ...) with
ctypes prototypes; :class:`SelSync` / :class:`Plan` wrap them with the same verbs
(``track_grad_change``, ``local_step``, ``aggregate_params``, ``step``).
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libselsync.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libselsync.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'` "
        "or `python paper_2307_07950_amd/build.py`. There is no CPU fallback." % LIB_PATH)

_lib = ctypes.CDLL(LIB_PATH)

SELSYNC_OK = 0
SELSYNC_ERR_INVALID_ARG = 1
SELSYNC_ERR_SHAPE_MISMATCH = 2
SELSYNC_ERR_DTYPE = 3
SELSYNC_ERR_OOM = 4
SELSYNC_ERR_HIP = 5
SELSYNC_ERR_NOT_DEVICE_MEM = 6
SELSYNC_ERR_STATE = 7
SELSYNC_ERR_TOO_LARGE = 8
SELSYNC_WARN_NONFINITE = 100
SELSYNC_F32 = 0
SELSYNC_BF16 = 1


class selsync_tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("numel", ctypes.c_int64), ("dtype", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class selsync_tensor_list(ctypes.Structure):
    _fields_ = [("tensors", ctypes.POINTER(selsync_tensor)), ("count", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class selsync_config(ctypes.Structure):
    _fields_ = [("num_workers", ctypes.c_int32), ("window", ctypes.c_int32), ("delta", ctypes.c_double),
                ("alpha", ctypes.c_double)]


class selsync_sgd(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("first_step", ctypes.c_int32), ("nesterov", ctypes.c_int32)]


class selsync_adam(ctypes.Structure):
    _fields_ = [("beta1", ctypes.c_double), ("beta2", ctypes.c_double), ("lr", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("grad_scale", ctypes.c_float),
                ("step", ctypes.c_int64)]


class selsync_stats(ctypes.Structure):
    _fields_ = [("steps_local", ctypes.c_int64), ("steps_sync", ctypes.c_int64), ("lssr", ctypes.c_double),
                ("max_delta", ctypes.c_double), ("nonfinite_steps", ctypes.c_int64)]


class selsync_tuning(ctypes.Structure):
    _fields_ = [("chunk_elems", ctypes.c_int32), ("nontemporal", ctypes.c_int32),
                ("agg_chunk_elems", ctypes.c_int32), ("ga_chunk_elems", ctypes.c_int32)]


_vp = ctypes.c_void_p
_i32 = ctypes.c_int32
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)
_tl = ctypes.POINTER(selsync_tensor_list)

# name -> (restype, argtypes); one entry per declaration in include/selsync.h
PROTOTYPES = {
    "selsync_create": (_i32, [ctypes.POINTER(selsync_config), ctypes.POINTER(_vp)]),
    "selsync_destroy": (_i32, [_vp]),
    "selsync_reset": (_i32, [_vp, _vp]),
    "selsync_set_delta": (_i32, [_vp, ctypes.c_double, _vp]),
    "selsync_set_tuning": (_i32, [_vp, ctypes.POINTER(selsync_tuning)]),
    "selsync_last_error": (ctypes.c_char_p, [_vp]),
    "selsync_status_string": (ctypes.c_char_p, [_i32]),
    "selsync_plan_create": (_i32, [_vp, _tl, _tl, _tl, _tl, _tl, _tl, ctypes.POINTER(_vp)]),
    "selsync_plan_destroy": (_i32, [_vp]),
    "selsync_plan_info": (_i32, [_vp, _ip, ctypes.POINTER(ctypes.c_int64), _ip, _ip]),
    "selsync_chunk_table_preview": (_i32, [ctypes.POINTER(ctypes.c_int64), _ip, _i32, _i32, _i32, _ip,
                                           ctypes.POINTER(ctypes.c_int64), _ip, _ip]),
    "selsync_track_grad_change": (_i32, [_vp, _vp, ctypes.c_float, _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_local_step": (_i32, [_vp, _vp, ctypes.POINTER(selsync_sgd), _vp]),
    "selsync_aggregate_params": (_i32, [_vp, _vp, _i32, _vp]),
    "selsync_step": (_i32, [_vp, _vp, ctypes.POINTER(selsync_sgd), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_step_bsp": (_i32, [_vp, _vp, ctypes.POINTER(selsync_sgd), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_plan_bind_second_moment": (_i32, [_vp, _tl]),
    "selsync_local_step_adam": (_i32, [_vp, _vp, ctypes.POINTER(selsync_adam), _vp]),
    "selsync_step_adam": (_i32, [_vp, _vp, ctypes.POINTER(selsync_adam), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_step_bsp_adam": (_i32, [_vp, _vp, ctypes.POINTER(selsync_adam), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_ga_update": (_i32, [_vp, _vp, ctypes.POINTER(selsync_sgd), _i32, _vp]),
    "selsync_step_ga": (_i32, [_vp, _vp, ctypes.POINTER(selsync_sgd), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_ga_update_adam": (_i32, [_vp, _vp, ctypes.POINTER(selsync_adam), _i32, _vp]),
    "selsync_step_ga_adam": (_i32, [_vp, _vp, ctypes.POINTER(selsync_adam), _vp, _i32, _dp, _dp, _ip, _ip]),
    "selsync_grad_norm_sq_noalloc": (_i32, [_tl, _i32, ctypes.c_float, _vp, _vp]),
    "selsync_partition_order": (_i32, [ctypes.c_int64, _i32, _i32, _i32, ctypes.c_int64,
                                       ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]),
    "selsync_partition_order_device": (_i32, [ctypes.c_int64, _i32, _i32, _i32, ctypes.c_int64, _vp,
                                              ctypes.POINTER(ctypes.c_int64), _vp]),
    "selsync_read_decision": (_i32, [_vp, _vp, _dp, _dp, _ip, _ip]),
    "selsync_read_tensor_norms": (_i32, [_vp, _vp, _vp, _dp]),
    "selsync_get_stats": (_i32, [_vp, _vp, ctypes.POINTER(selsync_stats)]),
    "selsync_tracker_state_size": (_i32, [_vp, ctypes.POINTER(ctypes.c_int64)]),
    "selsync_tracker_get_state": (_i32, [_vp, _vp, _vp, ctypes.c_int64]),
    "selsync_tracker_set_state": (_i32, [_vp, _vp, _vp, ctypes.c_int64]),
    "selsync_profile_enable": (_i32, [_vp, _i32, _i32]),
    "selsync_profile_config": (_i32, [_vp, _i32, _i32]),
    "selsync_profile_summary": (_i32, [_vp, _i32, ctypes.POINTER(ctypes.c_int64), _dp]),
}

for _name, (_res, _args) in PROTOTYPES.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args
    globals()[_name] = _fn


class SelSyncError(RuntimeError):
    def __init__(self, status: int, message: str):
        self.status = status
        super().__init__("%s: %s" % (_lib.selsync_status_string(status).decode(), message))


@dataclass
class Decision:
    norm_sq: List[float]
    delta: List[float]
    flags: List[int]
    sync: int
    nonfinite: bool = False


_DTYPES = {torch.float32: SELSYNC_F32, torch.bfloat16: SELSYNC_BF16}


def _stream_handle(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _marshal_lists(lists: Optional[Sequence[Sequence[torch.Tensor]]]):
    """[[tensor,...] per worker] -> (ctypes array of selsync_tensor_list, keep-alive objects)."""
    if lists is None:
        return None, []
    keep = []
    arr = (selsync_tensor_list * len(lists))()
    for k, tl in enumerate(lists):
        descs = (selsync_tensor * max(1, len(tl)))()
        for t, x in enumerate(tl):
            if not isinstance(x, torch.Tensor):
                raise TypeError("expected torch.Tensor")
            if not x.is_contiguous():
                raise ValueError("tensors must be contiguous")
            if x.dtype not in _DTYPES:
                raise TypeError("unsupported dtype %s" % x.dtype)
            descs[t].data = x.data_ptr() if x.numel() else None
            descs[t].numel = x.numel()
            descs[t].dtype = _DTYPES[x.dtype]
            descs[t].reserved = 0
        arr[k].tensors = descs
        arr[k].count = len(tl)
        arr[k].reserved = 0
        keep.append(descs)
        keep.append(list(tl))
    keep.append(arr)
    return arr, keep


def grad_norm_sq_noalloc(grads: Sequence[Sequence[torch.Tensor]], out: torch.Tensor, grad_scale: float = 1.0,
                         stream=None) -> None:
    """||grad_scale * g_k||^2 for every worker k into the float64 CUDA tensor `out` (one element per
    worker), through the entry point that allocates nothing (no context, no plan).  Asynchronous."""
    if out.dtype != torch.float64 or not out.is_cuda or not out.is_contiguous() or out.numel() != len(grads):
        raise ValueError("out must be a contiguous float64 CUDA tensor with one element per worker")
    arr, keep = _marshal_lists(grads)
    rc = selsync_grad_norm_sq_noalloc(arr, len(grads), grad_scale, _vp(out.data_ptr()), _vp(_stream_handle(stream)))
    if rc != SELSYNC_OK:
        raise SelSyncError(rc, "selsync_grad_norm_sq_noalloc")


def partition_order(num_samples: int, num_workers: int, worker: int, seldp: bool = True) -> List[int]:
    """Host-side reading order of one worker (DefDP or SelDP, Sec. III-D)."""
    n = ctypes.c_int64()
    rc = selsync_partition_order(num_samples, num_workers, worker, int(seldp), 0, None, ctypes.byref(n))
    if rc != SELSYNC_OK:
        raise SelSyncError(rc, "selsync_partition_order")
    out = (ctypes.c_int64 * max(1, n.value))()
    rc = selsync_partition_order(num_samples, num_workers, worker, int(seldp), n.value, out, ctypes.byref(n))
    if rc != SELSYNC_OK:
        raise SelSyncError(rc, "selsync_partition_order")
    return list(out)[:n.value]


def partition_order_device(num_samples: int, num_workers: int, worker: int, seldp: bool = True, stream=None):
    """The same order as an int64 CUDA tensor, produced by a kernel."""
    n = ctypes.c_int64()
    rc = selsync_partition_order(num_samples, num_workers, worker, int(seldp), 0, None, ctypes.byref(n))
    if rc != SELSYNC_OK:
        raise SelSyncError(rc, "selsync_partition_order")
    out = torch.empty(n.value, dtype=torch.int64, device="cuda")
    rc = selsync_partition_order_device(num_samples, num_workers, worker, int(seldp), n.value,
                                        _vp(out.data_ptr() if n.value else None), ctypes.byref(n),
                                        _vp(_stream_handle(stream)))
    if rc != SELSYNC_OK:
        raise SelSyncError(rc, "selsync_partition_order_device")
    return out


class Plan:
    """Chunk tables for one binding of tensor lists (selsync_plan)."""

    def __init__(self, owner: "SelSync", handle: int, keep):
        self._owner = owner
        self._h = _vp(handle)
        self._keep = keep          # the torch tensors must outlive the plan

    def info(self):
        t, p, uc, ac = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32()
        self._owner._check(selsync_plan_info(self._h, ctypes.byref(t), ctypes.byref(p), ctypes.byref(uc),
                                             ctypes.byref(ac)))
        return {"num_tensors": t.value, "num_params": p.value, "update_chunks": uc.value,
                "aggregate_chunks": ac.value}

    def destroy(self):
        if self._h is not None:
            selsync_plan_destroy(self._h)
            self._h = None
            self._keep = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class SelSync:
    """One selsync_ctx: K trackers + counters on the current GPU."""

    def __init__(self, num_workers: int, delta: float, window: int = 25, alpha: float = -1.0):
        if not torch.cuda.is_available():
            raise RuntimeError("SelSync needs a GPU; there is no CPU fallback")
        torch.cuda.init()
        torch.cuda.current_stream()    # make sure the HIP context of the current device exists
        cfg = selsync_config(num_workers, window, delta, alpha)
        h = _vp()
        rc = selsync_create(ctypes.byref(cfg), ctypes.byref(h))
        if rc != SELSYNC_OK:
            raise SelSyncError(rc, "selsync_create failed")
        self._h = h
        self.num_workers = num_workers
        self._plans: List[Plan] = []

    # -- helpers
    def _check(self, rc: int, allow_warn: bool = False) -> int:
        if rc == SELSYNC_OK or (allow_warn and rc == SELSYNC_WARN_NONFINITE):
            return rc
        raise SelSyncError(rc, selsync_last_error(self._h).decode())

    def _outs(self):
        K = self.num_workers
        return (ctypes.c_double * K)(), (ctypes.c_double * K)(), (ctypes.c_int32 * K)(), ctypes.c_int32()

    @staticmethod
    def _decision(rc, n, d, f, s) -> Decision:
        return Decision(list(n), list(d), list(f), s.value, rc == SELSYNC_WARN_NONFINITE)

    # -- lifecycle
    def set_tuning(self, chunk_elems: int = 0, nontemporal: int = -1, agg_chunk_elems: int = 0,
                   ga_chunk_elems: int = 0):
        t = selsync_tuning(chunk_elems, nontemporal, agg_chunk_elems, ga_chunk_elems)
        self._check(selsync_set_tuning(self._h, ctypes.byref(t)))

    def reset(self, stream=None):
        self._check(selsync_reset(self._h, _vp(_stream_handle(stream))))

    def set_delta(self, delta: float, stream=None):
        self._check(selsync_set_delta(self._h, delta, _vp(_stream_handle(stream))))

    def plan(self, grads, params, momenta, global_model, master=None, global_lowp=None) -> Plan:
        """grads/params/momenta/master: K lists of tensors; global_model/global_lowp: one list.
        ``momenta=None`` with gradients given makes a momentum-free plan (plain SGD only)."""
        for name, lists in (("grads", grads), ("params", params), ("momenta", momenta), ("master", master)):
            if lists is not None and len(lists) != self.num_workers:
                raise ValueError("%s: expected %d lists (one per worker), got %d"
                                 % (name, self.num_workers, len(lists)))
        keep = []
        arrs = []
        for lists in (grads, params, momenta, master,
                      None if global_model is None else [global_model],
                      None if global_lowp is None else [global_lowp]):
            a, k = _marshal_lists(lists)
            arrs.append(a)
            keep.append(k)
        h = _vp()
        self._check(selsync_plan_create(self._h, arrs[0], arrs[1], arrs[2], arrs[3], arrs[4], arrs[5],
                                        ctypes.byref(h)))
        p = Plan(self, h.value, keep)
        self._plans.append(p)
        return p

    # -- per-step path (same verbs as the C entry points)
    def track_grad_change(self, plan: Plan, grad_scale: float = 1.0, blocking: bool = True, stream=None):
        n, d, f, s = self._outs()
        rc = self._check(selsync_track_grad_change(self._h, plan._h, grad_scale, _vp(_stream_handle(stream)),
                                                   int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    def local_step(self, plan: Plan, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                   grad_scale: float = 1.0, first_step: int = -1, stream=None, nesterov: bool = False):
        sgd = selsync_sgd(lr, momentum, weight_decay, grad_scale, first_step, int(nesterov))
        self._check(selsync_local_step(self._h, plan._h, ctypes.byref(sgd), _vp(_stream_handle(stream))))

    def aggregate_params(self, plan: Plan, always: bool = False, stream=None):
        self._check(selsync_aggregate_params(self._h, plan._h, 1 if always else 0, _vp(_stream_handle(stream))))

    def step(self, plan: Plan, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
             grad_scale: float = 1.0, first_step: int = -1, blocking: bool = False, stream=None,
             nesterov: bool = False):
        sgd = selsync_sgd(lr, momentum, weight_decay, grad_scale, first_step, int(nesterov))
        n, d, f, s = self._outs()
        rc = self._check(selsync_step(self._h, plan._h, ctypes.byref(sgd), _vp(_stream_handle(stream)),
                                      int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    def step_bsp(self, plan: Plan, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                 grad_scale: float = 1.0, first_step: int = -1, blocking: bool = False, stream=None,
                 nesterov: bool = False):
        """One fully synchronous iteration in a single pass: update, tracking and unconditional aggregation."""
        sgd = selsync_sgd(lr, momentum, weight_decay, grad_scale, first_step, int(nesterov))
        n, d, f, s = self._outs()
        rc = self._check(selsync_step_bsp(self._h, plan._h, ctypes.byref(sgd), _vp(_stream_handle(stream)),
                                          int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    # -- variant: Adam local update
    def bind_second_moment(self, plan: Plan, second_moment):
        if len(second_moment) != self.num_workers:
            raise ValueError("expected %d lists" % self.num_workers)
        arr, keep = _marshal_lists(second_moment)
        self._check(selsync_plan_bind_second_moment(plan._h, arr))
        plan._keep.append(keep)

    def local_step_adam(self, plan: Plan, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                        weight_decay: float = 0.0, grad_scale: float = 1.0, step: int = 0, stream=None):
        ad = selsync_adam(beta1, beta2, lr, eps, weight_decay, grad_scale, step)
        self._check(selsync_local_step_adam(self._h, plan._h, ctypes.byref(ad), _vp(_stream_handle(stream))))

    def step_adam(self, plan: Plan, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                  weight_decay: float = 0.0, grad_scale: float = 1.0, step: int = 0, blocking: bool = False,
                  stream=None):
        ad = selsync_adam(beta1, beta2, lr, eps, weight_decay, grad_scale, step)
        n, d, f, s = self._outs()
        rc = self._check(selsync_step_adam(self._h, plan._h, ctypes.byref(ad), _vp(_stream_handle(stream)),
                                           int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    def step_bsp_adam(self, plan: Plan, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                      weight_decay: float = 0.0, grad_scale: float = 1.0, step: int = 0, blocking: bool = False,
                      stream=None):
        ad = selsync_adam(beta1, beta2, lr, eps, weight_decay, grad_scale, step)
        n, d, f, s = self._outs()
        rc = self._check(selsync_step_bsp_adam(self._h, plan._h, ctypes.byref(ad), _vp(_stream_handle(stream)),
                                               int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    # -- variant: gradient aggregation
    def ga_update(self, plan: Plan, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                  grad_scale: float = 1.0, first_step: int = -1, always: bool = False, stream=None,
                  nesterov: bool = False):
        sgd = selsync_sgd(lr, momentum, weight_decay, grad_scale, first_step, int(nesterov))
        self._check(selsync_ga_update(self._h, plan._h, ctypes.byref(sgd), 1 if always else 0,
                                      _vp(_stream_handle(stream))))

    def step_ga(self, plan: Plan, lr: float, momentum: float = 0.0, weight_decay: float = 0.0,
                grad_scale: float = 1.0, first_step: int = -1, blocking: bool = False, stream=None,
                nesterov: bool = False):
        sgd = selsync_sgd(lr, momentum, weight_decay, grad_scale, first_step, int(nesterov))
        n, d, f, s = self._outs()
        rc = self._check(selsync_step_ga(self._h, plan._h, ctypes.byref(sgd), _vp(_stream_handle(stream)),
                                         int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    def ga_update_adam(self, plan: Plan, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                       weight_decay: float = 0.0, grad_scale: float = 1.0, step: int = 0, always: bool = False,
                       stream=None):
        ad = selsync_adam(beta1, beta2, lr, eps, weight_decay, grad_scale, step)
        self._check(selsync_ga_update_adam(self._h, plan._h, ctypes.byref(ad), 1 if always else 0,
                                           _vp(_stream_handle(stream))))

    def step_ga_adam(self, plan: Plan, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                     weight_decay: float = 0.0, grad_scale: float = 1.0, step: int = 0, blocking: bool = False,
                     stream=None):
        ad = selsync_adam(beta1, beta2, lr, eps, weight_decay, grad_scale, step)
        n, d, f, s = self._outs()
        rc = self._check(selsync_step_ga_adam(self._h, plan._h, ctypes.byref(ad), _vp(_stream_handle(stream)),
                                              int(blocking), n, d, f, ctypes.byref(s)), allow_warn=True)
        return self._decision(rc, n, d, f, s) if blocking else None

    # -- observability
    def read_decision(self, stream=None) -> Decision:
        n, d, f, s = self._outs()
        rc = self._check(selsync_read_decision(self._h, _vp(_stream_handle(stream)), n, d, f, ctypes.byref(s)),
                         allow_warn=True)
        return self._decision(rc, n, d, f, s)

    def read_tensor_norms(self, plan: Plan, stream=None) -> List[List[float]]:
        """[k][t] squared norms of the last tracking pass on `plan`."""
        T = plan.info()["num_tensors"]
        out = (ctypes.c_double * max(1, self.num_workers * T))()
        self._check(selsync_read_tensor_norms(self._h, plan._h, _vp(_stream_handle(stream)), out))
        return [[out[k * T + t] for t in range(T)] for k in range(self.num_workers)]

    def stats(self, stream=None) -> dict:
        st = selsync_stats()
        self._check(selsync_get_stats(self._h, _vp(_stream_handle(stream)), ctypes.byref(st)))
        return {"steps_local": st.steps_local, "steps_sync": st.steps_sync, "lssr": st.lssr,
                "max_delta": st.max_delta, "nonfinite_steps": st.nonfinite_steps}

    def get_state(self, stream=None) -> bytes:
        n = ctypes.c_int64()
        self._check(selsync_tracker_state_size(self._h, ctypes.byref(n)))
        buf = ctypes.create_string_buffer(n.value)
        self._check(selsync_tracker_get_state(self._h, _vp(_stream_handle(stream)), buf, n.value))
        return buf.raw

    def set_state(self, blob: bytes, stream=None):
        buf = ctypes.create_string_buffer(blob, len(blob))
        self._check(selsync_tracker_set_state(self._h, _vp(_stream_handle(stream)), buf, len(blob)))

    def profile_enable(self, enable: bool = True, max_launches: int = 4096):
        self._check(selsync_profile_enable(self._h, int(enable), max_launches))

    def profile_config(self, kind_mask: int = 7, stride: int = 1):
        self._check(selsync_profile_config(self._h, kind_mask, stride))

    def profile_summary(self, kind: int):
        c, ms = ctypes.c_int64(), ctypes.c_double()
        self._check(selsync_profile_summary(self._h, kind, ctypes.byref(c), ctypes.byref(ms)))
        return c.value, ms.value

    def close(self):
        if self._h is not None:
            for p in self._plans:
                p.destroy()
            self._plans = []
            selsync_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
