"""ctypes front-end of the plain-C SelSync oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this.
It never touches the GPU library and shares no code with it.  All arithmetic lives
in ``selsync_oracle.c``; this file only builds it with gcc, marshals numpy arrays
and strings the four per-step operations together in the order of Alg. 1:

    for every worker:  x = ||g||^2 (line 8) -> local update (line 9) -> Delta, flag (lines 8, 10-11)
    any flag set (lines 12-13)  ->  parameter aggregation (lines 14-15)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "selsync_oracle.c")
_LIB = os.path.join(_HERE, "libselsync_oracle.so")

CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no FMA contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        f32p = ctypes.POINTER(ctypes.c_float)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        L.selsync_oracle_bf16_to_f32.restype = ctypes.c_float
        L.selsync_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.selsync_oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.selsync_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        L.selsync_oracle_norm_sq_accum_f32.restype = ctypes.c_double
        L.selsync_oracle_norm_sq_accum_f32.argtypes = [ctypes.c_double, f32p, ctypes.c_int64, ctypes.c_float]
        L.selsync_oracle_norm_sq_accum_bf16.restype = ctypes.c_double
        L.selsync_oracle_norm_sq_accum_bf16.argtypes = [ctypes.c_double, u16p, ctypes.c_int64, ctypes.c_float]
        L.selsync_oracle_sgd_f32.restype = None
        L.selsync_oracle_sgd_f32.argtypes = [f32p, f32p, f32p, ctypes.c_int64] + [ctypes.c_float] * 4 + [ctypes.c_int]
        L.selsync_oracle_sgd_bf16.restype = None
        L.selsync_oracle_sgd_bf16.argtypes = [f32p, f32p, u16p, u16p, ctypes.c_int64] + [ctypes.c_float] * 4 + [ctypes.c_int]
        L.selsync_oracle_average_f32.restype = None
        L.selsync_oracle_sgd_plain_f32.argtypes = [f32p, f32p, ctypes.c_int64] + [ctypes.c_float] * 3
        L.selsync_oracle_sgd_plain_f32.restype = None
        L.selsync_oracle_sgd_plain_bf16.argtypes = [f32p, u16p, u16p, ctypes.c_int64] + [ctypes.c_float] * 3
        L.selsync_oracle_sgd_plain_bf16.restype = None
        L.selsync_oracle_sgd_nesterov_f32.argtypes = [f32p, f32p, f32p, ctypes.c_int64] + [ctypes.c_float] * 4 + [ctypes.c_int]
        L.selsync_oracle_sgd_nesterov_f32.restype = None
        L.selsync_oracle_sgd_nesterov_bf16.argtypes = [f32p, f32p, u16p, u16p, ctypes.c_int64] + [ctypes.c_float] * 4 + [ctypes.c_int]
        L.selsync_oracle_sgd_nesterov_bf16.restype = None
        L.selsync_oracle_average_f32.argtypes = [ctypes.POINTER(f32p), ctypes.c_int, f32p, ctypes.c_int64]
        L.selsync_oracle_average_bf16.restype = None
        L.selsync_oracle_average_bf16.argtypes = [ctypes.POINTER(f32p), ctypes.POINTER(u16p), ctypes.c_int,
                                                  f32p, u16p, ctypes.c_int64]
        L.selsync_oracle_average_grads_f32.restype = None
        L.selsync_oracle_average_grads_f32.argtypes = [ctypes.POINTER(f32p), ctypes.c_int, ctypes.c_float, f32p,
                                                       ctypes.c_int64]
        L.selsync_oracle_average_grads_bf16.restype = None
        L.selsync_oracle_average_grads_bf16.argtypes = [ctypes.POINTER(u16p), ctypes.c_int, ctypes.c_float, f32p,
                                                        ctypes.c_int64]
        L.selsync_oracle_adam_f32.restype = None
        L.selsync_oracle_adam_f32.argtypes = [f32p, f32p, f32p, f32p, ctypes.c_int64] + [ctypes.c_float] * 10 + [ctypes.c_int]
        L.selsync_oracle_adam_bf16.restype = None
        L.selsync_oracle_adam_bf16.argtypes = [f32p, f32p, f32p, u16p, u16p, ctypes.c_int64] + [ctypes.c_float] * 10 + [ctypes.c_int]
        L.selsync_oracle_tracker_new.restype = ctypes.c_void_p
        L.selsync_oracle_tracker_new.argtypes = [ctypes.c_int, ctypes.c_double]
        L.selsync_oracle_tracker_free.restype = None
        L.selsync_oracle_tracker_free.argtypes = [ctypes.c_void_p]
        L.selsync_oracle_tracker_push.restype = ctypes.c_double
        L.selsync_oracle_tracker_push.argtypes = [ctypes.c_void_p, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
        L.selsync_oracle_flag.restype = ctypes.c_int
        L.selsync_oracle_flag.argtypes = [ctypes.c_double, ctypes.c_double]
        _lib = L
    return _lib


def _f32(a: np.ndarray):
    assert a.dtype == np.float32 and a.flags.c_contiguous, (a.dtype, a.flags.c_contiguous)
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u16(a: np.ndarray):
    assert a.dtype == np.uint16 and a.flags.c_contiguous, (a.dtype, a.flags.c_contiguous)
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


# ---------------------------------------------------------------- scalar helpers

def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen an array of bf16 bit patterns (uint16) to fp32, element by element."""
    L = lib()
    flat = np.ascontiguousarray(bits, dtype=np.uint16).ravel()
    out = np.empty(flat.shape, dtype=np.float32)
    for i, h in enumerate(flat):
        out[i] = L.selsync_oracle_bf16_to_f32(int(h))
    return out.reshape(np.shape(bits))


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round an fp32 array to bf16 bit patterns (uint16), nearest-even."""
    L = lib()
    flat = np.ascontiguousarray(x, dtype=np.float32).ravel()
    out = np.empty(flat.shape, dtype=np.uint16)
    for i, v in enumerate(flat):
        out[i] = L.selsync_oracle_f32_to_bf16(float(v))
    return out.reshape(np.shape(x))


# ---------------------------------------------------------------- a1

def norm_sq(tensors: Sequence[np.ndarray], grad_scale: float = 1.0) -> float:
    """||g||^2 over a whole tensor list, fp64, flat index order (Alg. 1 line 8)."""
    L = lib()
    acc = 0.0
    for g in tensors:
        if g.dtype == np.float32:
            acc = L.selsync_oracle_norm_sq_accum_f32(acc, _f32(g), g.size, grad_scale)
        elif g.dtype == np.uint16:
            acc = L.selsync_oracle_norm_sq_accum_bf16(acc, _u16(g), g.size, grad_scale)
        else:
            raise TypeError("gradient must be float32 or bf16 bits in uint16, got %s" % g.dtype)
    return acc


# ---------------------------------------------------------------- a3

def sgd_update(params: Sequence[np.ndarray], momenta: Optional[Sequence[np.ndarray]], grads: Sequence[np.ndarray],
               lr: float, momentum: float, weight_decay: float, grad_scale: float = 1.0, first: bool = False,
               copies: Optional[Sequence[np.ndarray]] = None, nesterov: bool = False) -> None:
    """In-place local update of one replica (Alg. 1 line 9).  With ``copies`` the
    gradients are bf16 bits, ``params`` are the fp32 masters and ``copies`` receive
    the bf16-rounded parameters.  ``momenta=None`` is momentum-free SGD (no buffer;
    ``momentum`` must be 0); ``nesterov`` selects the look-ahead step direction."""
    L = lib()
    if momenta is None:
        assert momentum == 0.0 and not nesterov
        for t, (w, g) in enumerate(zip(params, grads)):
            assert w.size == g.size
            if copies is None:
                L.selsync_oracle_sgd_plain_f32(_f32(w), _f32(g), w.size, lr, weight_decay, grad_scale)
            else:
                assert copies[t].size == w.size
                L.selsync_oracle_sgd_plain_bf16(_f32(w), _u16(g), _u16(copies[t]), w.size, lr, weight_decay, grad_scale)
        return
    f32_fn = L.selsync_oracle_sgd_nesterov_f32 if nesterov else L.selsync_oracle_sgd_f32
    bf16_fn = L.selsync_oracle_sgd_nesterov_bf16 if nesterov else L.selsync_oracle_sgd_bf16
    for t, (w, m, g) in enumerate(zip(params, momenta, grads)):
        assert w.size == m.size == g.size
        if copies is None:
            f32_fn(_f32(w), _f32(m), _f32(g), w.size, lr, momentum, weight_decay, grad_scale, int(first))
        else:
            c = copies[t]
            assert c.size == w.size
            bf16_fn(_f32(w), _f32(m), _u16(g), _u16(c), w.size, lr, momentum, weight_decay, grad_scale, int(first))


# ---------------------------------------------------------------- a4

def average_params(replicas: Sequence[Sequence[np.ndarray]], global_model: Sequence[np.ndarray],
                   copies: Optional[Sequence[Sequence[np.ndarray]]] = None,
                   global_copy: Optional[Sequence[np.ndarray]] = None) -> None:
    """Mean over the K replicas into the global model and back into every replica
    (Alg. 1 lines 14-15).  ``replicas[k][t]`` is tensor t of worker k."""
    L = lib()
    K = len(replicas)
    f32p = ctypes.POINTER(ctypes.c_float)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    for t in range(len(global_model)):
        n = global_model[t].size
        ptrs = (f32p * K)(*[_f32(replicas[k][t]) for k in range(K)])
        for k in range(K):
            assert replicas[k][t].size == n
        if copies is None:
            L.selsync_oracle_average_f32(ptrs, K, _f32(global_model[t]), n)
        else:
            cptrs = (u16p * K)(*[_u16(copies[k][t]) for k in range(K)])
            L.selsync_oracle_average_bf16(ptrs, cptrs, K, _f32(global_model[t]), _u16(global_copy[t]), n)


# ---------------------------------------------------------------- variant: Adam local update

def adam_constants(beta1: float, beta2: float, step: int):
    """(omb1, omb2, bc1, bc2) as the fp32 values the update uses: 1-beta and the bias
    corrections 1-beta^t of step t (1-based), formed in double and rounded once."""
    b1, b2 = float(beta1), float(beta2)        # the betas are double-precision inputs
    return (float(np.float32(1.0 - b1)), float(np.float32(1.0 - b2)),
            float(np.float32(1.0 - b1 ** step)), float(np.float32(1.0 - b2 ** step)))


def adam_update(params, m, v, grads, lr, beta1, beta2, eps, weight_decay, step: int, grad_scale: float = 1.0,
                copies=None) -> None:
    """In-place Adam update of one replica at 1-based step `step` (Sec. IV-A, AlexNet recipe)."""
    L = lib()
    omb1, omb2, bc1, bc2 = adam_constants(beta1, beta2, step)
    for t in range(len(params)):
        n = params[t].size
        if copies is None:
            L.selsync_oracle_adam_f32(_f32(params[t]), _f32(m[t]), _f32(v[t]), _f32(grads[t]), n, lr, beta1, beta2,
                                      omb1, omb2, eps, weight_decay, grad_scale, bc1, bc2, int(step == 1))
        else:
            L.selsync_oracle_adam_bf16(_f32(params[t]), _f32(m[t]), _f32(v[t]), _u16(grads[t]), _u16(copies[t]), n,
                                       lr, beta1, beta2, omb1, omb2, eps, weight_decay, grad_scale, bc1, bc2,
                                       int(step == 1))


# ---------------------------------------------------------------- variant: gradient aggregation

def average_grads(grads: Sequence[Sequence[np.ndarray]], grad_scale: float = 1.0) -> List[np.ndarray]:
    """Mean over the K workers of the scaled gradients, one fp32 array per tensor (Sec. III-C)."""
    L = lib()
    K = len(grads)
    f32p = ctypes.POINTER(ctypes.c_float)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    out = []
    for t in range(len(grads[0])):
        n = grads[0][t].size
        gbar = np.empty(n, np.float32)
        if grads[0][t].dtype == np.uint16:
            ptrs = (u16p * K)(*[_u16(grads[k][t]) for k in range(K)])
            L.selsync_oracle_average_grads_bf16(ptrs, K, grad_scale, _f32(gbar), n)
        else:
            ptrs = (f32p * K)(*[_f32(grads[k][t]) for k in range(K)])
            L.selsync_oracle_average_grads_f32(ptrs, K, grad_scale, _f32(gbar), n)
        out.append(gbar)
    return out


def ga_update(grads, params, momenta, lr, momentum, weight_decay, grad_scale=1.0, first=False, sync=True,
              copies=None, nesterov=False) -> None:
    """Update of all K workers under gradient aggregation (Sec. III-C): on a synchronising step every
    worker applies the averaged gradient to its own state, otherwise its own gradient.  ``momenta=None``
    is momentum-free SGD.  In mixed precision (``copies`` given) the averaged fp32 gradient acts on the
    fp32 masters and every bf16 copy is then refreshed by rounding its master."""
    K = len(params)
    mom = lambda k: None if momenta is None else momenta[k]
    if not sync:
        for k in range(K):
            sgd_update(params[k], mom(k), grads[k], lr, momentum, weight_decay, grad_scale, first,
                       None if copies is None else copies[k], nesterov=nesterov)
        return
    gbar = average_grads(grads, grad_scale)
    for k in range(K):
        sgd_update(params[k], mom(k), gbar, lr, momentum, weight_decay, 1.0, first, nesterov=nesterov)
        if copies is not None:
            for t in range(len(gbar)):
                copies[k][t][...] = f32_to_bf16(params[k][t])


def ga_update_adam(grads, params, m, v, lr, beta1, beta2, eps, weight_decay, step: int, grad_scale=1.0, sync=True,
                   copies=None) -> None:
    """Gradient aggregation with Adam as the update (Sec. III-C with the Adam recipe of Sec. IV-A): on a
    synchronising step every worker feeds the averaged gradient to its OWN Adam state (both moment
    buffers stay per worker), otherwise its own gradient.  `step` is the 1-based step of the bias
    corrections, the same for every worker."""
    K = len(params)
    if not sync:
        for k in range(K):
            adam_update(params[k], m[k], v[k], grads[k], lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                        None if copies is None else copies[k])
        return
    gbar = average_grads(grads, grad_scale)
    for k in range(K):
        adam_update(params[k], m[k], v[k], gbar, lr, beta1, beta2, eps, weight_decay, step, 1.0)
        if copies is not None:
            for t in range(len(gbar)):
                copies[k][t][...] = f32_to_bf16(params[k][t])


# ---------------------------------------------------------------- a2

class Tracker:
    """One worker's RelativeGradChange state (Eq. 2 with windowed EWMA smoothing)."""

    def __init__(self, window: int = 25, alpha: float = 0.16):
        self._L = lib()
        self._h = self._L.selsync_oracle_tracker_new(window, alpha)
        if not self._h:
            raise ValueError("window must be >= 1")
        self.window, self.alpha = window, alpha
        self.smoothed = float("nan")

    def push(self, x: float) -> float:
        s = ctypes.c_double()
        d = self._L.selsync_oracle_tracker_push(self._h, float(x), ctypes.byref(s))
        self.smoothed = s.value
        return d

    def __del__(self):
        try:
            self._L.selsync_oracle_tracker_free(self._h)
        except Exception:
            pass


def flag(delta_g: float, threshold: float) -> int:
    return lib().selsync_oracle_flag(delta_g, threshold)


# ---------------------------------------------------------------- data partitioning (Sec. III-D)

def partition_chunks(num_samples: int, num_workers: int):
    """Split sample indices 0..D-1 into N contiguous chunks DP0..DP(N-1) of (near-)equal size:
    the first D mod N chunks hold one sample more."""
    base, rem = divmod(num_samples, num_workers)
    chunks, start = [], 0
    for c in range(num_workers):
        size = base + (1 if c < rem else 0)
        chunks.append(list(range(start, start + size)))
        start += size
    return chunks


def defdp_order(num_samples: int, num_workers: int, worker: int):
    """Default partitioning: worker n only ever sees its own chunk DPn."""
    return partition_chunks(num_samples, num_workers)[worker]


def seldp_order(num_samples: int, num_workers: int, worker: int):
    """SelSync partitioning: every worker sees ALL chunks, as a circular queue whose head is
    rotated to the worker's own chunk: worker n reads DPn, DP(n+1), ..., DP(n-1)."""
    chunks = partition_chunks(num_samples, num_workers)
    order = []
    for j in range(num_workers):
        order.extend(chunks[(worker + j) % num_workers])
    return order


# ---------------------------------------------------------------- one whole step

@dataclass
class StepRecord:
    norm_sq: List[float]
    delta: List[float]
    flags: List[int]
    sync: int


@dataclass
class OracleSelSync:
    """K workers' trackers plus the step/sync counters (LSSR, Eq. 4)."""
    num_workers: int
    delta: float
    window: int = 25
    alpha: float = -1.0            # <= 0: min(1, num_workers / 100) (smoothing factor N/100, Sec. III-A)
    steps_local: int = 0
    steps_sync: int = 0
    max_delta: float = 0.0
    steps_done: int = 0
    trackers: List[Tracker] = field(default_factory=list)

    def __post_init__(self):
        if self.alpha <= 0:
            # N/100 is stated for N = 16; a smoothing factor lies in (0, 1], so beyond 100 workers it stays 1
            self.alpha = min(1.0, self.num_workers / 100.0)
        self.trackers = [Tracker(self.window, self.alpha) for _ in range(self.num_workers)]

    def track(self, grads: Sequence[Sequence[np.ndarray]], grad_scale: float = 1.0) -> StepRecord:
        """a1 + a2 for every worker, then the any-worker rule (Sec. III-B)."""
        return self.track_norms([norm_sq(grads[k], grad_scale) for k in range(self.num_workers)])

    def track_norms(self, norms: Sequence[float]) -> StepRecord:
        """a2 for every worker from this iteration's ||g_k||^2, then the any-worker rule (Sec. III-B)."""
        xs, ds, fs = [], [], []
        for k in range(self.num_workers):
            x = float(norms[k])
            d = self.trackers[k].push(x)
            xs.append(x)
            ds.append(d)
            fs.append(flag(d, self.delta))
            if np.isfinite(d):
                self.max_delta = max(self.max_delta, d)
        sync = int(any(fs))
        self.steps_sync += sync
        self.steps_local += 1 - sync
        return StepRecord(xs, ds, fs, sync)

    def step(self, grads, params, momenta, global_model, lr, momentum, weight_decay, grad_scale=1.0,
             copies=None, global_copy=None, first: Optional[bool] = None,
             force_sync: Optional[int] = None) -> StepRecord:
        """One iteration of Alg. 1 for all K workers held in host memory.

        ``force_sync`` lets a parity harness impose a decision when the statistic
        sits within the stated tolerance of the threshold."""
        if first is None:
            first = self.steps_done == 0
        rec = self.track(grads, grad_scale)
        for k in range(self.num_workers):
            sgd_update(params[k], momenta[k], grads[k], lr, momentum, weight_decay, grad_scale, first,
                       None if copies is None else copies[k])
        do_sync = rec.sync if force_sync is None else force_sync
        if do_sync:
            average_params(params, global_model, copies, global_copy)
        self.steps_done += 1
        return rec

    @property
    def lssr(self) -> float:
        tot = self.steps_local + self.steps_sync
        return self.steps_local / tot if tot else float("nan")
