"""Seeded synthetic workloads: tensor shapes and gradient/parameter generators.

This module holds NO arithmetic of the method (no norm, no tracker, no update, no
averaging).  It only says what the tensors look like and fills them with seeded
random numbers on the host, so that the CPU oracle and the GPU library can be fed
bit-identical inputs.  Shapes follow the four model families of the paper's
evaluation (Sec. IV-A: ResNet101, VGG11, AlexNet, Transformer) plus a tiny MLP;
the real datasets and trained weights are not available, so gradients are random
draws whose scale follows a schedule with the qualitative behaviour of Fig. 5
(large changes early, decay, isolated spikes).

Gradient sets are unit-scale draws Z[k][b] (worker k, pool slot b); step t uses
slot ``t % pool`` multiplied by the scalar ``sigma(t)`` -- passed to the library as
``grad_scale`` -- so hundreds of full-size steps do not need hundreds of full-size
random draws.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]


def _numel(s: Shape) -> int:
    n = 1
    for d in s:
        n *= d
    return n


# --------------------------------------------------------------------------- shapes

def mlp_shapes() -> List[Shape]:
    return [(784, 256), (256,), (256, 256), (256,), (256, 10), (10,)]


def resnet_shapes(width: int = 64, num_classes: int = 1000) -> List[Shape]:
    """Bottleneck ResNet, stage depths [3, 4, 23, 3], expansion 4, 3x3 stem.

    Every convolution is followed by a BN scale vector and a BN shift vector; the
    first block of each stage has a 1x1 down-sample convolution (+BN)."""
    shapes: List[Shape] = []

    def conv_bn(cout, cin, k):
        shapes.append((cout, cin, k, k))
        shapes.append((cout,))
        shapes.append((cout,))

    conv_bn(width, 3, 3)
    cin = width
    for stage, depth in enumerate([3, 4, 23, 3]):
        mid = width * (2 ** stage)
        out = mid * 4
        for b in range(depth):
            conv_bn(mid, cin, 1)
            conv_bn(mid, mid, 3)
            conv_bn(out, mid, 1)
            if b == 0:
                conv_bn(out, cin, 1)
            cin = out
    shapes.append((num_classes, cin))
    shapes.append((num_classes,))
    return shapes


def alexnet_shapes(div: int = 1) -> List[Shape]:
    c = lambda x: max(1, x // div)
    convs = [(c(64), 3, 11, 11), (c(192), c(64), 5, 5), (c(384), c(192), 3, 3), (c(256), c(384), 3, 3),
             (c(256), c(256), 3, 3)]
    shapes: List[Shape] = []
    for s in convs:
        shapes += [s, (s[0],)]
    fcs = [(c(4096), c(256) * 36), (c(4096), c(4096)), (1000, c(4096))]
    for s in fcs:
        shapes += [s, (s[0],)]
    return shapes


def vgg11_shapes(div: int = 1) -> List[Shape]:
    c = lambda x: max(1, x // div)
    chans = [3, c(64), c(128), c(256), c(256), c(512), c(512), c(512), c(512)]
    shapes: List[Shape] = []
    for i in range(8):
        shapes += [(chans[i + 1], chans[i], 3, 3), (chans[i + 1],)]
    fcs = [(c(4096), c(512) * 49), (c(4096), c(4096)), (1000, c(4096))]
    for s in fcs:
        shapes += [s, (s[0],)]
    return shapes


def transformer_shapes(d: int = 512, ffn: int = 2048, vocab: int = 33278, layers: int = 6) -> List[Shape]:
    """Encoder-decoder stack, `layers` of each, tied embedding and an output bias."""
    shapes: List[Shape] = []

    def attn():
        shapes.extend([(3 * d, d), (3 * d,), (d, d), (d,)])

    def ln():
        shapes.extend([(d,), (d,)])

    def mlp():
        shapes.extend([(ffn, d), (ffn,), (d, ffn), (d,)])

    for _ in range(layers):           # encoder layer
        attn(); ln(); mlp(); ln()
    ln()
    for _ in range(layers):           # decoder layer: self-attn, cross-attn, ffn
        attn(); ln(); attn(); ln(); mlp(); ln()
    ln()
    shapes.append((vocab, d))
    shapes.append((vocab,))
    return shapes


# --------------------------------------------------------------------------- workloads

@dataclass
class Workload:
    name: str
    shapes: List[Shape]
    num_workers: int                 # K replicas
    steps: int
    delta: float                     # sync threshold
    lr: float
    momentum: float
    weight_decay: float
    seed: int
    mixed_bf16: bool = False         # bf16 grads + bf16 param copy, fp32 master/momentum
    window: int = 25
    pool: int = 2                    # B unit-scale gradient sets per worker
    param_std: float = 0.05
    grad_dist: str = "normal"        # "normal" | "student_t3"
    unit_scale: float = 1.0          # multiplies the unit draws when they are generated
    per_tensor_log_range: float = 0.0   # >0: per-tensor factor log-uniform in [10^-r, 10^r]
    bn_like_init: bool = False       # 1-D tensors come in (scale, shift) pairs initialised to 1 / 0
    sigma: Callable[[int], float] = field(default=lambda t: 1.0)
    description: str = ""

    @property
    def numels(self) -> List[int]:
        return [_numel(s) for s in self.shapes]

    @property
    def num_params(self) -> int:
        return sum(self.numels)

    @property
    def num_tensors(self) -> int:
        return len(self.shapes)

    def sigmas(self, steps: int = None) -> List[float]:
        return [float(np.float32(self.sigma(t))) for t in range(self.steps if steps is None else steps)]


def _rng(seed: int, *stream: int) -> np.random.Generator:
    """Counter-based generator keyed by (seed, stream ids...): every tensor of every
    worker/slot has its own reproducible stream, independent of generation order."""
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, *[int(s) for s in stream]])))


def _lognormal_decay_schedule(seed: int, steps: int, tau: float = 100.0, jitter: float = 0.25,
                              base: float = 1e-2) -> List[float]:
    xi = _rng(seed, 7777).standard_normal(steps)
    return [base * math.exp(-t / tau + jitter * float(xi[t])) for t in range(steps)]


def get(name: str, shrink: int = 1, steps: int = None, num_workers: int = None) -> Workload:
    """Return one of the five workloads.  ``shrink`` divides channel widths so the
    oracle can run many steps in seconds; ``shrink=1`` is the full-size model."""
    name = name.lower()
    if name in ("c1", "mlp", "tiny_mlp"):
        spikes = (10, 30)
        wl = Workload("tiny_mlp", mlp_shapes(), 4, 50, 0.3, 0.1, 0.9, 5e-4, seed=0, pool=50,
                      sigma=lambda t: 1e-2 * (0.98 ** t) * (3.0 if t in spikes else 1.0),
                      description="6-tensor MLP, grads N(0,1e-2) drifting 0.98x/step, 3x spike at steps 10 and 30")
    elif name in ("c2", "resnet", "resnet_like"):
        nsteps = 200
        sched = _lognormal_decay_schedule(1, 4096)
        wl = Workload("resnet_like", resnet_shapes(max(4, 64 // shrink)), 8, nsteps, 0.3, 0.1, 0.9, 4e-4, seed=1,
                      bn_like_init=True, sigma=lambda t: sched[t % len(sched)],
                      description="bottleneck ResNet [3,4,23,3], 314 tensors, grads N(0,sigma_t), log-normal decay")
    elif name in ("c3", "alexnet", "alexnet_like"):
        wl = Workload("alexnet_like", alexnet_shapes(shrink), 8, 200, 0.3, 0.01, 0.9, 5e-4, seed=2,
                      grad_dist="student_t3", unit_scale=1e-3, sigma=lambda t: 1.0,
                      description="AlexNet-shaped, 16 tensors, heavy-tailed grads (Student-t df=3, scale 1e-3)")
    elif name in ("c4", "vgg11", "vgg11_like"):
        wl = Workload("vgg11_like", vgg11_shapes(shrink), 4, 200, 0.3, 0.01, 0.9, 5e-4, seed=3,
                      sigma=lambda t: 1e-3 * (4.0 if (t > 0 and t % 25 == 0) else 1.0),
                      description="VGG11-shaped, 22 tensors, grads N(0,1e-3), 4x spike every 25 steps")
    elif name in ("c5", "transformer", "transformer_like"):
        d = max(16, 512 // shrink)
        wl = Workload("transformer_like", transformer_shapes(d, 4 * d, max(64, 33278 // (shrink * shrink))), 8,
                      500, 0.1, 0.05, 0.9, 0.0, seed=4, mixed_bf16=True, param_std=0.02, unit_scale=1e-3,
                      per_tensor_log_range=1.0, sigma=lambda t: 1.0,
                      description="6+6 layer Transformer LM shape, bf16 grads/params with fp32 master, "
                                  "per-tensor grad scale spanning 100x")
    else:
        raise KeyError(name)
    if steps is not None:
        wl.steps = steps
    if num_workers is not None:
        wl.num_workers = num_workers
    return wl


FULL_SIZE_PARAMS: Dict[str, Tuple[int, int]] = {      # name -> (tensors, parameters) at shrink=1
    "tiny_mlp": (6, 269_322),
    "resnet_like": (314, 44_541_480),
    "alexnet_like": (16, 61_100_840),
    "vgg11_like": (22, 132_863_336),
    "transformer_like": (186, 61_212_158),
}


# --------------------------------------------------------------------------- bf16 storage helper

def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Storage-format conversion for generated inputs: fp32 -> bf16 bit patterns,
    nearest-even (finite inputs only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- generators

def initial_params(wl: Workload) -> List[np.ndarray]:
    """One replica's initial fp32 parameters (all K replicas start identical: every
    worker pulls the same initial state).  In mixed mode the values are the fp32
    masters; the bf16 copies are their nearest-even roundings."""
    out = []
    one_d = 0
    for t, n in enumerate(wl.numels):
        if wl.bn_like_init and len(wl.shapes[t]) == 1 and t < len(wl.shapes) - 1:
            out.append(np.full(n, 1.0 if one_d % 2 == 0 else 0.0, dtype=np.float32))
            one_d += 1
            continue
        r = _rng(wl.seed, 1, t)
        out.append((r.standard_normal(n, dtype=np.float32) * np.float32(wl.param_std)).astype(np.float32))
    return out


def tensor_factors(wl: Workload) -> List[float]:
    if wl.per_tensor_log_range <= 0:
        return [1.0] * wl.num_tensors
    r = _rng(wl.seed, 2)
    e = r.uniform(-wl.per_tensor_log_range, wl.per_tensor_log_range, wl.num_tensors)
    return [float(10.0 ** v) for v in e]


def unit_grads(wl: Workload, worker: int, slot: int) -> List[np.ndarray]:
    """Gradient set Z[worker][slot]: fp32 arrays, or bf16 bit patterns (uint16) in mixed mode."""
    fac = tensor_factors(wl)
    out = []
    for t, n in enumerate(wl.numels):
        r = _rng(wl.seed, 3, worker, slot, t)
        if wl.grad_dist == "normal":
            z = r.standard_normal(n, dtype=np.float32)
        elif wl.grad_dist == "student_t3":
            z = r.standard_t(3.0, n).astype(np.float32)
        else:
            raise ValueError(wl.grad_dist)
        z = (z * np.float32(wl.unit_scale * fac[t])).astype(np.float32)
        out.append(round_to_bf16_bits(z) if wl.mixed_bf16 else z)
    return out
