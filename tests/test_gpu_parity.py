"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Bars: ||g||^2 within 1e-5 relative; updated
parameters / momenta within 1 fp32 ulp; averaged parameters within 1e-6 relative;
decisions identical unless |Delta - delta| <= 1e-5."""
import ctypes
import math
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import selsync_oracle as O                          # noqa: E402
from paper_2307_07950_amd import workloads as W                 # noqa: E402
from tests import parity_util as PU                             # noqa: E402


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding
    return binding


def rng(seed):
    return np.random.default_rng(seed)


SMALL_CHUNK = dict(chunk_elems=8192, nontemporal=1)   # pieces of 32 tiles: the multi-tile loop of the streaming kernel

# tensor-size sets: tiny / ragged tails / several tiles / empty tensors / exactly one chunk
SIZE_SETS = {
    "tiny": [1, 2, 3, 5, 10],
    "ragged": [4097, 8191, 8193, 65537, 7, 1023],
    "tiles": [3 * 65536 + 13, 65536, 2 * 8192],
    "with_empty": [0, 100, 0, 70000, 0],
    "one": [123457],
}


# ================================================================= a1: squared norm

@pytest.mark.parametrize("sizes", list(SIZE_SETS))
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1, 3])
def test_norm_matches_oracle(B, sizes, mixed, misalign):
    numel = SIZE_SETS[sizes]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.3, mixed=mixed, misalign=misalign, tuning=SMALL_CHUNK, seed=1)
    r = rng(10)
    grads = []
    for k in range(K):
        gk = [(r.standard_normal(n) * 10.0 ** r.uniform(-4, 1)).astype(np.float32) for n in numel]
        grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
    ls.bind_grads(0, grads)
    for gs in (1.0, 0.37):
        dec = ls.ctx.track_grad_change(ls.plans[0], gs, blocking=True)
        for k in range(K):
            want = O.norm_sq(grads[k], gs)
            assert dec.norm_sq[k] == pytest.approx(want, rel=PU.NORM_RTOL)
            assert dec.norm_sq[k] == pytest.approx(want, rel=1e-12)      # fp64 accumulation: far inside the bar
    ls.close()


def test_norm_invariants_zero_constant_and_determinism(B):
    numel = [100000, 33, 70001]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=0.3, tuning=SMALL_CHUNK)
    c = 0.5
    ls.bind_grads(0, [[np.zeros(n, np.float32) for n in numel], [np.full(n, c, np.float32) for n in numel]])
    dec = ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    assert dec.norm_sq[0] == 0.0
    assert dec.norm_sq[1] == sum(numel) * c * c
    # run-to-run bitwise determinism on random data (no atomics, fixed slots, fixed order)
    r = rng(3)
    g = [[r.standard_normal(n).astype(np.float32) for n in numel] for _ in range(K)]
    ls.bind_grads(1, g)
    first = ls.ctx.track_grad_change(ls.plans[1], 1.0, blocking=True).norm_sq
    for _ in range(5):
        again = ls.ctx.track_grad_change(ls.plans[1], 1.0, blocking=True).norm_sq
        assert [x.hex() for x in again] == [x.hex() for x in first]
    ls.close()


def test_norm_nonfinite_gradient_sets_flag_and_warns(B):
    numel = [5000, 9000]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=float("inf"))
    r = rng(4)
    g = [[r.standard_normal(n).astype(np.float32) for n in numel] for _ in range(K)]
    g[1][1][77] = np.inf
    ls.bind_grads(0, g)
    dec = ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    rec = ls.oracle.track(g, 1.0)
    assert dec.nonfinite and dec.flags == [0, 1, 0] == rec.flags and dec.sync == 1 == rec.sync
    assert math.isinf(dec.delta[1]) and math.isinf(rec.delta[1])
    assert ls.ctx.stats()["nonfinite_steps"] == 1
    ls.close()


# ================================================================= a3: local update

@pytest.mark.parametrize("sizes", list(SIZE_SETS))
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1])
def test_local_step_matches_oracle_over_steps(B, sizes, mixed, misalign):
    numel = SIZE_SETS[sizes]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=float("inf"), mixed=mixed, misalign=misalign, tuning=SMALL_CHUNK, seed=2)
    r = rng(20)
    for slot in range(2):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    for t in range(6):
        ls.step(t % 2, lr=0.1, mu=0.9, wd=5e-4, gs=[1.0, 0.5, 1.7][t % 3], fused=(t % 2 == 0))
    assert ls.worst_ulp == 0          # same rounding sequence on both sides: bit-identical in practice
    ls.close()


@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("phase_w,phase_g", [(0, 1), (2, 0), (1, 3), (3, 3), (2, 2)])
def test_streams_at_different_address_phases(B, mixed, phase_w, phase_g):
    # equal phases: head peel + 128-bit body; different phases: the element-wise path.  Same results.
    numel = [70001, 5, 4096, 2, 1023]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=0.0, mixed=mixed, misalign=phase_w, misalign_g=phase_g, seed=23)
    r = rng(25)
    grads = []
    for k in range(K):
        gk = [(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel]
        grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
    ls.bind_grads(0, grads)
    for t in range(3):
        ls.step(0, lr=0.1, mu=0.9, wd=5e-4, gs=0.9, fused=(t != 1))      # delta 0: every step also aggregates
    ls.steps_done = 0
    ls.step_ga(0, 0.1, 0.9, 5e-4, 0.9)
    assert ls.worst_ulp == 0
    ls.close()


def test_local_step_lr_zero_is_noop_and_plain_sgd_special_case(B):
    numel = [40000, 17]
    ls = PU.LockStep(B, numel, 1, delta=float("inf"), seed=5)
    r = rng(21)
    g = [[r.standard_normal(n).astype(np.float32) for n in numel]]
    ls.bind_grads(0, g)
    w0 = [PU.to_host(t) for t in ls.d_w[0]]
    ls.ctx.local_step(ls.plans[0], lr=0.0, momentum=0.9, weight_decay=5e-4, first_step=1)
    for t in range(len(numel)):
        assert PU.to_host(ls.d_w[0][t]).tobytes() == w0[t].tobytes()
    # momentum 0, weight decay 0: w - lr*g exactly (Alg. 1 line 9)
    ls.ctx.local_step(ls.plans[0], lr=0.25, momentum=0.0, weight_decay=0.0, first_step=0)
    for t in range(len(numel)):
        want = (w0[t].astype(np.float64) - (np.float32(0.25) * g[0][t]).astype(np.float64)).astype(np.float32)
        assert PU.to_host(ls.d_w[0][t]).tobytes() == want.tobytes()
    ls.close()


def test_local_step_automatic_first_step(B):
    numel = [1000]
    ls = PU.LockStep(B, numel, 1, delta=float("inf"), seed=6)
    g = [[rng(22).standard_normal(1000).astype(np.float32)]]
    ls.bind_grads(0, g)
    ls.d_m[0][0].fill_(1e6)                      # garbage momentum must be ignored on the first step
    ls.ctx.local_step(ls.plans[0], lr=0.1, momentum=0.9, weight_decay=0.0, first_step=-1)
    assert PU.to_host(ls.d_m[0][0]).tobytes() == g[0][0].tobytes()
    ls.ctx.local_step(ls.plans[0], lr=0.1, momentum=0.9, weight_decay=0.0, first_step=-1)
    want = (np.float32(0.9) * g[0][0]) + g[0][0]
    assert PU.to_host(ls.d_m[0][0]).tobytes() == want.tobytes()
    ls.ctx.reset()
    ls.ctx.local_step(ls.plans[0], lr=0.1, momentum=0.9, weight_decay=0.0, first_step=-1)
    assert PU.to_host(ls.d_m[0][0]).tobytes() == g[0][0].tobytes()
    ls.close()


@pytest.mark.parametrize("mixed", [False, True])
def test_many_chunks_take_the_segment_reduction_level(B, mixed):
    # more than 16384 chunks: per-chunk partials -> per-segment sums -> tracker
    numel = [4_200_000 + 13, 77]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=float("inf"), mixed=mixed, seed=3)
    r = rng(23)
    grads = []
    for k in range(K):
        gk = [(r.standard_normal(n, dtype=np.float32) * np.float32(1e-2)) for n in numel]
        grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
    ls.bind_grads(0, grads)
    assert ls.plans[0].info()["update_chunks"] > 16384
    for t in range(2):
        ls.step(0, lr=0.1, mu=0.9, wd=5e-4, gs=1.0 + t, fused=(t == 0))
    assert ls.worst_norm_rel < 1e-12 and ls.worst_ulp == 0
    ls.close()


@pytest.mark.parametrize("chunk", [0, 256, 768, 1024, 2048, 65536])
@pytest.mark.parametrize("nt", [0, 1])
def test_every_piece_size_and_access_kind_gives_the_same_results(B, chunk, nt):
    numel = [100003, 513, 4096, 255]
    K = 2
    tuning = dict(chunk_elems=chunk, nontemporal=nt)
    for mixed in (False, True):
        ls = PU.LockStep(B, numel, K, delta=0.0, mixed=mixed, tuning=tuning, seed=4)
        r = rng(24)
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(0, grads)
        for t in range(3):
            ls.step(0, lr=0.1, mu=0.9, wd=5e-4, gs=1.0, fused=(t != 1))
        assert ls.worst_ulp == 0
        ls.close()


# ================================================================= a4: aggregation

@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 8, 16])
@pytest.mark.parametrize("mixed", [False, True])
def test_aggregate_matches_oracle(B, K, mixed):
    numel = [70001, 5, 8192, 0, 33333]
    ls = PU.LockStep(B, numel, K, delta=0.0, mixed=mixed, tuning=SMALL_CHUNK, seed=7)
    r = rng(30 + K)
    # make the replicas differ
    for k in range(K):
        for t, n in enumerate(numel):
            pert = (r.standard_normal(n) * 1e-3).astype(np.float32)
            ls.h_w[k][t] += pert
            ls.d_w[k][t].copy_(torch.from_numpy(ls.h_w[k][t]))
    m_before = [[PU.to_host(x) for x in ls.d_m[k]] for k in range(K)]
    ls.bind_grads(0, [[W.round_to_bf16_bits(np.zeros(n, np.float32)) if mixed else np.zeros(n, np.float32)
                       for n in numel] for _ in range(K)])
    pre = [np.max(np.abs(np.stack([ls.h_w[k][t] for k in range(K)])), axis=0).astype(np.float64)
           for t in range(len(numel))]
    ls.ctx.aggregate_params(ls.plans[0], always=True)
    O.average_params(ls.h_w, ls.h_glob, ls.h_c, ls.h_gc)
    ls._pre_scale = pre
    ls.compare(after_sync=True)
    for t in range(len(numel)):      # fp64 sum in the same order on both sides: expect identical bits
        assert PU.to_host(ls.d_glob[t]).tobytes() == ls.h_glob[t].tobytes()
    for k in range(K):               # momentum untouched
        for t in range(len(numel)):
            assert PU.to_host(ls.d_m[k][t]).tobytes() == m_before[k][t].tobytes()
    ls.close()


@pytest.mark.parametrize("chunk", [256, 512, 768, 1024, 4096, 8192])
@pytest.mark.parametrize("K", [3, 4])
def test_aggregate_piece_sizes_give_identical_results(B, chunk, K):
    # the table of the decision-following launch, cut into pieces of the given size (one-wavefront
    # workgroups below 1024 elements, 256-thread workgroups from there on)
    numel = [70001, 5, 8192, 0, 33333]
    for mixed in (False, True):
        ls = PU.LockStep(B, numel, K, delta=0.3, mixed=mixed, seed=7,
                         tuning=dict(agg_chunk_elems=chunk, nontemporal=K % 2))
        r = rng(300 + K)
        for k in range(K):
            for t, n in enumerate(numel):
                ls.h_w[k][t] += (r.standard_normal(n) * 1e-3).astype(np.float32)
                ls.d_w[k][t].copy_(torch.from_numpy(ls.h_w[k][t]))
        grads = []
        for k in range(K):
            gk = [r.standard_normal(n).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(0, grads)
        # a 3x jump of the gradient scale makes the device-side decision "sync" under delta = 0.3
        assert ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True).sync == 0
        assert ls.ctx.track_grad_change(ls.plans[0], 3.0, blocking=True).sync == 1
        ls.ctx.aggregate_params(ls.plans[0], always=False)
        O.average_params(ls.h_w, ls.h_glob, ls.h_c, ls.h_gc)
        for t in range(len(numel)):
            assert PU.to_host(ls.d_glob[t]).tobytes() == ls.h_glob[t].tobytes()
            if mixed:
                assert PU.to_host(ls.d_gc[t]).tobytes() == ls.h_gc[t].tobytes()
            for k in range(K):
                assert PU.to_host(ls.d_w[k][t]).tobytes() == ls.h_w[k][t].tobytes()
                if mixed:
                    assert PU.to_host(ls.d_c[k][t]).tobytes() == ls.h_c[k][t].tobytes()
        ls.close()


def test_aggregate_identical_replicas_is_identity_and_misaligned(B):
    numel = [10001, 64, 3]
    K = 4
    ls = PU.LockStep(B, numel, K, delta=0.0, misalign=1, seed=8)
    ls.bind_grads(0, [[np.zeros(n, np.float32) for n in numel] for _ in range(K)])
    ls.ctx.aggregate_params(ls.plans[0], always=True)
    for t in range(len(numel)):
        assert PU.to_host(ls.d_glob[t]).tobytes() == ls.h_w[0][t].tobytes()
        for k in range(K):
            assert PU.to_host(ls.d_w[k][t]).tobytes() == ls.h_w[0][t].tobytes()
    ls.close()


def test_aggregate_mode0_follows_device_decision(B):
    numel = [50000]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=float("inf"), seed=9)
    ls.d_w[1][0].add_(1.0)
    before = [PU.to_host(ls.d_w[k][0]) for k in range(K)]
    g = [[rng(40 + k).standard_normal(50000).astype(np.float32)] for k in range(K)]
    ls.bind_grads(0, g)
    dec = ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    assert dec.sync == 0
    ls.ctx.aggregate_params(ls.plans[0], always=False)          # decision is "local": nothing may change
    for k in range(K):
        assert PU.to_host(ls.d_w[k][0]).tobytes() == before[k].tobytes()
    assert not PU.to_host(ls.d_glob[0]).any()
    ls.ctx.set_delta(0.0)
    dec = ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    assert dec.sync == 1
    ls.ctx.aggregate_params(ls.plans[0], always=False)
    want = ((before[0].astype(np.float64) + before[1].astype(np.float64)) / 2).astype(np.float32)
    assert PU.to_host(ls.d_glob[0]).tobytes() == want.tobytes()
    ls.close()


def test_threshold_zero_aggregates_every_tracked_step_but_not_before_the_first_decision(B):
    # delta = 0 turns SelSync into BSP (Sec. III-B): every tracked step synchronises.  Before any
    # tracking call there is no decision yet, so a predicated aggregation does nothing.
    numel = [50000, 7]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.0, seed=61)
    for k in range(K):
        ls.d_w[k][0].add_(float(k))
    before = [[PU.to_host(x) for x in ls.d_w[k]] for k in range(K)]
    ls.bind_grads(0, [[rng(400 + k).standard_normal(n).astype(np.float32) for n in numel] for k in range(K)])
    ls.ctx.aggregate_params(ls.plans[0], always=False)
    for k in range(K):
        for t in range(len(numel)):
            assert PU.to_host(ls.d_w[k][t]).tobytes() == before[k][t].tobytes()
    dec = ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    assert dec.sync == 1
    ls.ctx.aggregate_params(ls.plans[0], always=False)
    want = (sum(b[0].astype(np.float64) for b in before) / K).astype(np.float32)
    for k in range(K):
        assert PU.to_host(ls.d_w[k][0]).tobytes() == want.tobytes()
    assert PU.to_host(ls.d_glob[0]).tobytes() == want.tobytes()
    ls.ctx.reset()
    ls.d_w[1][1].add_(1.0)
    snap = PU.to_host(ls.d_w[1][1])
    ls.ctx.aggregate_params(ls.plans[0], always=False)          # after a reset there is again no decision
    assert PU.to_host(ls.d_w[1][1]).tobytes() == snap.tobytes()
    ls.close()


# ================================================================= a2 + whole steps

def test_fused_step_is_bit_identical_to_three_calls(B):
    numel = [100003, 257, 65536]
    K = 4
    r = rng(50)
    runs = []
    for fused in (True, False):
        ls = PU.LockStep(B, numel, K, delta=0.05, alpha=0.5, window=5, tuning=SMALL_CHUNK, seed=11)
        rr = rng(51)
        for slot in range(3):
            ls.bind_grads(slot, [[(rr.standard_normal(n) * (1 + slot)).astype(np.float32) for n in numel]
                                 for _ in range(K)])
        decs = []
        for t in range(9):
            dec, _ = ls.step(t % 3, 0.05, 0.9, 1e-4, 1.0, fused=fused)
            decs.append(dec)
        state = [[PU.to_host(x).tobytes() for x in ls.d_w[k]] + [PU.to_host(x).tobytes() for x in ls.d_m[k]]
                 for k in range(K)]
        runs.append((decs, state, [PU.to_host(x).tobytes() for x in ls.d_glob]))
        assert ls.oracle.steps_sync > 0 and ls.oracle.steps_local > 0
        ls.close()
    (d1, s1, g1), (d2, s2, g2) = runs
    assert s1 == s2 and g1 == g2
    for a, b in zip(d1, d2):
        assert a.flags == b.flags and a.sync == b.sync
        assert [x.hex() for x in a.norm_sq] == [x.hex() for x in b.norm_sq]
        assert [x.hex() for x in a.delta] == [x.hex() for x in b.delta]


@pytest.mark.parametrize("window,alpha", [(1, 0.16), (25, 0.04), (25, 1.0), (200, 0.16), (3, 0.5), (2048, 0.01)])
def test_tracker_matches_oracle_for_windows_and_alphas(B, window, alpha):
    numel = [3000]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=0.05, window=window, alpha=alpha, seed=12)
    g = [[rng(60 + k).standard_normal(3000).astype(np.float32)] for k in range(K)]
    ls.bind_grads(0, g)
    r = rng(61)
    nsteps = 2 * window + 10 if window <= 25 else window + 30
    scales = np.exp(np.cumsum(r.standard_normal(nsteps) * 0.15))
    for t in range(nsteps):
        ls.step(0, 0.0, 0.0, 0.0, float(np.float32(scales[t])), compare_tensors=False)
    assert ls.oracle.steps_sync > 0 and ls.oracle.steps_local > 0
    st = ls.ctx.stats()
    assert st["max_delta"] == pytest.approx(ls.oracle.max_delta, rel=1e-9)
    ls.close()


def test_the_largest_window_a_context_accepts(B):
    # 65536 is the limit of selsync_create; the window never fills here, the state only has to be laid out for it
    with pytest.raises(B.SelSyncError):
        B.SelSync(2, 0.3, window=65537)
    ls = PU.LockStep(B, [3000], 2, delta=0.05, window=65536, alpha=0.3, seed=15)
    ls.bind_grads(0, [[rng(65 + k).standard_normal(3000).astype(np.float32)] for k in range(2)])
    for t, gs in enumerate([1.0, 1.0, 1.5, 1.5, 0.7, 0.7, 0.7, 2.0]):
        ls.step(0, 0.01, 0.9, 0.0, gs)
    assert ls.oracle.steps_sync > 0 and ls.oracle.steps_local > 0
    blob = ls.ctx.get_state()                          # the checkpoint carries the whole (mostly empty) window
    assert len(blob) > 2 * 65536 * 8
    ls.close()


def test_delta_zero_is_bsp_and_huge_delta_is_local_only_on_gpu(B):
    numel = [20000, 31]
    K = 3
    for delta, lssr in ((0.0, 0.0), (float("inf"), 1.0)):
        ls = PU.LockStep(B, numel, K, delta=delta, seed=13)
        for slot in range(2):
            ls.bind_grads(slot, [[rng(70 + 10 * slot + k).standard_normal(n).astype(np.float32) for n in numel]
                                 for k in range(K)])
        for t in range(8):
            dec, _ = ls.step(t % 2, 0.1, 0.9, 1e-4)
            assert dec.sync == (1 if delta == 0.0 else 0)
        assert ls.ctx.stats()["lssr"] == lssr
        ls.close()


def test_reset_clears_tracker_and_counters(B):
    numel = [4096]
    ls = PU.LockStep(B, numel, 2, delta=0.0, seed=14)
    ls.bind_grads(0, [[rng(80 + k).standard_normal(4096).astype(np.float32)] for k in range(2)])
    for _ in range(3):
        ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True)
    assert ls.ctx.stats()["steps_sync"] == 3
    ls.ctx.reset()
    st = ls.ctx.stats()
    assert st["steps_sync"] == 0 and st["steps_local"] == 0 and math.isnan(st["lssr"])
    dec = ls.ctx.track_grad_change(ls.plans[0], 3.0, blocking=True)
    assert dec.delta == [0.0, 0.0]               # no previous smoothed value again
    ls.close()


def test_per_tensor_norms_match_oracle(B):
    numel = [70001, 0, 5, 4096, 513]
    K = 3
    for mixed in (False, True):
        ls = PU.LockStep(B, numel, K, delta=0.3, mixed=mixed, seed=17)
        r = rng(97)
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 10.0 ** r.uniform(-3, 0)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(0, grads)
        with pytest.raises(B.SelSyncError) as e:
            ls.ctx.read_tensor_norms(ls.plans[0])
        assert e.value.status == B.SELSYNC_ERR_STATE
        dec = ls.ctx.track_grad_change(ls.plans[0], 0.5, blocking=True)
        got = ls.ctx.read_tensor_norms(ls.plans[0])
        for k in range(K):
            for t in range(len(numel)):
                want = O.norm_sq([grads[k][t]], 0.5)
                assert got[k][t] == pytest.approx(want, rel=1e-12, abs=0.0)
            assert sum(got[k]) == pytest.approx(dec.norm_sq[k], rel=1e-12)
        ls.close()


def test_tracker_state_checkpoint_and_resume(B):
    numel = [9000]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=0.05, window=7, alpha=0.3, seed=18)
    g = [[rng(98 + k).standard_normal(9000).astype(np.float32)] for k in range(K)]
    ls.bind_grads(0, g)
    scales = [float(np.float32(v)) for v in np.exp(np.cumsum(rng(99).standard_normal(30) * 0.2))]
    for t in range(12):
        ls.ctx.track_grad_change(ls.plans[0], scales[t], blocking=True)
    blob = ls.ctx.get_state()
    stats_at_save = ls.ctx.stats()
    tail_a = [ls.ctx.track_grad_change(ls.plans[0], scales[t], blocking=True) for t in range(12, 30)]
    # a fresh context with the same configuration resumes from the blob
    ctx2 = B.SelSync(K, 0.9, 7, 0.3)                 # different delta: the blob restores it
    plan2 = ctx2.plan(ls.d_grads[0], ls.d_w, ls.d_m, ls.d_glob)
    ctx2.set_state(blob)
    assert ctx2.stats() == stats_at_save
    tail_b = [ctx2.track_grad_change(plan2, scales[t], blocking=True) for t in range(12, 30)]
    for a, b in zip(tail_a, tail_b):
        assert a.flags == b.flags and a.sync == b.sync
        assert [x.hex() for x in a.delta] == [x.hex() for x in b.delta]
    assert ctx2.stats() == ls.ctx.stats()
    # a context with another window refuses the blob
    ctx3 = B.SelSync(K, 0.05, 8, 0.3)
    with pytest.raises(B.SelSyncError) as e:
        ctx3.set_state(blob)
    assert e.value.status == B.SELSYNC_ERR_INVALID_ARG
    ctx3.close()
    ctx2.close()
    ls.close()


def test_checkpoint_restores_the_threshold_on_host_and_device(B):
    """A blob saved under delta = 0.3 restored into a context that was created with delta = 0 and has
    already taken a decision: from then on the context must behave as under 0.3 (local steps are NOT
    averaged), checked against the oracle on decisions and every tensor."""
    numel = [70001, 513, 4096]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.3, window=5, alpha=0.5, seed=71)
    r = rng(710)
    for slot in range(2):
        ls.bind_grads(slot, [[(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
                             for _ in range(K)])
    sched = [0, 0, 1, 1, 0, 0, 1, 0, 1, 1, 0, 0]
    for t in range(5):
        ls.step(sched[t], 0.05, 0.9, 1e-4, 1.0)
    blob = ls.ctx.get_state()
    ctx2 = B.SelSync(K, 0.0, 5, 0.5)
    plans2 = {slot: ctx2.plan(ls.d_grads[slot], ls.d_w, ls.d_m, ls.d_glob) for slot in (0, 1)}
    assert ctx2.track_grad_change(plans2[0], 1.0, blocking=True).sync == 1     # delta 0: "every step syncs"
    ctx2.set_state(blob)
    assert ctx2.stats() == ls.ctx.stats()
    old = ls.ctx
    ls.ctx, ls.plans = ctx2, plans2
    syncs = 0
    for t in range(5, 12):
        dec, rec = ls.step(sched[t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
        syncs += rec.sync
    assert 0 < syncs < 7 and ls.worst_ulp == 0 and ls.forced == 0
    # the gradient-aggregation update takes the same host-side shortcut: it must follow the decision too
    for t in range(3):
        ls.step_ga(sched[t], 0.05, 0.9, 1e-4, 1.0, fused=(t != 1))
    # and the other direction: a delta = 0 blob restored into a delta = 0.3 context synchronises every step
    ctx3 = B.SelSync(K, 0.0, 5, 0.5)
    ctx3.track_grad_change(ctx3.plan(ls.d_grads[0], ls.d_w, ls.d_m, ls.d_glob), 1.0, blocking=True)
    blob0 = ctx3.get_state()
    ctx3.close()
    ls.ctx.set_state(blob0)
    ls.oracle = O.OracleSelSync(K, 0.0, 5, 0.5)
    ls.oracle.track(ls.h_grads[0], 1.0)
    for t in range(3):
        dec, rec = ls.step(sched[t], 0.05, 0.9, 1e-4, 1.0, fused=(t != 1))
        assert dec.sync == 1
    assert ls.worst_ulp == 0
    old.close()
    ls.close()


def test_mode0_follows_the_device_decision_after_the_threshold_changes(B):
    """The decision of the last tracking call stands until the next one: lowering delta to 0 after a
    "local" decision must not make a mode-0 aggregation (or gradient-aggregation update) synchronise."""
    numel = [50000, 7]
    K = 2
    ls = PU.LockStep(B, numel, K, delta=0.3, seed=72)
    ls.d_w[1][0].add_(1.0)
    ls.h_w[1][0] += np.float32(1.0)
    before = [[PU.to_host(x) for x in ls.d_w[k]] for k in range(K)]
    ls.bind_grads(0, [[rng(720 + k).standard_normal(n).astype(np.float32) for n in numel] for k in range(K)])
    assert ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True).sync == 0
    ls.oracle.track(ls.h_grads[0], 1.0)
    ls.ctx.set_delta(0.0)
    ls.ctx.aggregate_params(ls.plans[0], always=False)
    for k in range(K):
        for t in range(len(numel)):
            assert PU.to_host(ls.d_w[k][t]).tobytes() == before[k][t].tobytes()
    assert not PU.to_host(ls.d_glob[0]).any()
    # same for the gradient-aggregation update: the decision is "local", each worker applies its own gradient
    ls.ctx.ga_update(ls.plans[0], 0.1, 0.9, 1e-4, 1.0, first_step=1, always=False)
    O.ga_update(ls.h_grads[0], ls.h_w, ls.h_m, 0.1, 0.9, 1e-4, 1.0, True, False)
    ls.compare()
    # the next tracking call decides under the new threshold
    assert ls.ctx.track_grad_change(ls.plans[0], 1.0, blocking=True).sync == 1
    ls.ctx.aggregate_params(ls.plans[0], always=False)
    O.average_params(ls.h_w, ls.h_glob)
    for t in range(len(numel)):
        assert PU.to_host(ls.d_glob[t]).tobytes() == ls.h_glob[t].tobytes()
    ls.close()


@pytest.mark.parametrize("variant,K,mixed", [("pa", 4, False), ("ga", 4, False), ("ga", 3, True), ("pa", 3, True),
                                             ("ga_adam", 4, False), ("ga_adam", 3, True), ("pa_adam", 4, True)])
def test_graph_captured_at_threshold_zero_follows_a_later_threshold(B, variant, K, mixed):
    """A step recorded into a HIP graph under delta = 0 (when the library expects every step to
    synchronise) and replayed after selsync_set_delta(0.3) must take the decisions of delta = 0.3:
    every replay is compared with the oracle, decisions and tensors."""
    numel = [150001, 777, 4096]
    r = rng(730)
    ls = PU.LockStep(B, numel, K, delta=0.0, window=4, alpha=0.5, seed=73, mixed=mixed)
    g0 = [[(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel] for _ in range(K)]
    ls.bind_grads(0, [[W.round_to_bf16_bits(a) for a in gk] for gk in g0] if mixed else g0)
    scales = [1.0, 1.0, 4.0, 1.0, 1.0, 0.25, 1.0]           # powers of two: exact in bf16 as well
    adam = variant.endswith("_adam")
    AD = (1e-3, 0.9, 0.999, 1e-8, 1e-2)                      # lr, betas, eps, weight decay of the Adam variants
    if adam:
        ls.enable_adam()
        (ls.step_adam if variant == "pa_adam" else ls.step_ga_adam)(0, *AD, scales[0])
    else:
        (ls.step if variant == "pa" else ls.step_ga)(0, 0.05, 0.9, 1e-4, scales[0])   # eager, delta = 0: synchronises
    assert ls.oracle.steps_sync == 1
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        if variant == "pa":
            ls.ctx.step(ls.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=0)
        elif variant == "ga":
            ls.ctx.step_ga(ls.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=0)
        elif variant == "pa_adam":                           # the bias-correction step is recorded with the launch:
            ls.ctx.step_adam(ls.plans[0], *AD, 1.0, step=2)  # every replay is "step 2", on both sides
        else:
            ls.ctx.step_ga_adam(ls.plans[0], *AD, 1.0, step=2)
    ls.ctx.set_delta(0.3)
    ls.oracle.delta = 0.3
    syncs = 0
    for t in range(1, 7):
        for k in range(K):                                  # eager work between replays: rescale the gradients
            for i, x in enumerate(ls.d_grads[0][k]):
                f = np.float32(scales[t]) / np.float32(scales[t - 1])
                x.mul_(float(f))
                if mixed:
                    ls.h_grads[0][k][i][...] = W.round_to_bf16_bits(W.bf16_bits_to_f32(ls.h_grads[0][k][i]) * f)
                else:
                    ls.h_grads[0][k][i] *= f
        g.replay()
        torch.cuda.synchronize()
        dec = ls.ctx.read_decision()
        rec = ls.oracle.track(ls.h_grads[0], 1.0)
        sync = ls._check_decision(dec, rec)
        assert ls.forced == 0
        if variant == "pa":
            for k in range(K):
                O.sgd_update(ls.h_w[k], ls.h_m[k], ls.h_grads[0][k], 0.05, 0.9, 1e-4, 1.0, False,
                             None if not mixed else ls.h_c[k])
            if sync:
                O.average_params(ls.h_w, ls.h_glob, ls.h_c, ls.h_gc)
        elif variant == "ga":
            O.ga_update(ls.h_grads[0], ls.h_w, ls.h_m, 0.05, 0.9, 1e-4, 1.0, False, bool(sync), ls.h_c)
        elif variant == "pa_adam":
            for k in range(K):
                O.adam_update(ls.h_w[k], ls.h_m[k], ls.h_v[k], ls.h_grads[0][k], *AD, 2, 1.0,
                              None if not mixed else ls.h_c[k])
            if sync:
                O.average_params(ls.h_w, ls.h_glob, ls.h_c, ls.h_gc)
        else:
            O.ga_update_adam(ls.h_grads[0], ls.h_w, ls.h_m, ls.h_v, *AD, 2, 1.0, bool(sync), ls.h_c)
        ls.steps_done += 1
        ls.compare()
        if adam:
            for k in range(K):
                for i in range(len(numel)):
                    assert PU.to_host(ls.d_v[k][i]).tobytes() == ls.h_v[k][i].tobytes()
        if variant.startswith("pa") and sync:
            for t2 in range(len(numel)):
                assert PU.to_host(ls.d_glob[t2]).tobytes() == ls.h_glob[t2].tobytes()
        syncs += sync
    assert 0 < syncs < 6 and ls.worst_ulp == 0
    del g
    ls.close()


def test_step_can_be_captured_in_a_hip_graph_and_replayed(B):
    """selsync_step neither allocates nor synchronises, so a caller may capture it.  Every replay
    (with eager work and synchronisations between replays) must equal the eager run bit for bit."""
    numel = [150001, 777, 4096]
    K = 4
    r = rng(150)
    grads = [[(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel] for _ in range(K)]
    scales = [1.0, 1.0, 3.0, 1.0, 1.0, 0.2, 1.0]

    def fresh():
        ls = PU.LockStep(B, numel, K, delta=0.2, window=4, alpha=0.5, seed=22)
        ls.bind_grads(0, grads)
        return ls

    # eager reference: step 0 with first_step=1, then 6 identical-argument steps (grad_scale via the tensor below)
    eager = fresh()
    eager.ctx.step(eager.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=1)
    decs_e = []
    for t in range(6):
        for k in range(K):                       # eager work between steps: rescale worker gradients in place
            for x in eager.d_grads[0][k]:
                x.mul_(scales[t + 1] / scales[t])
        decs_e.append(eager.ctx.step(eager.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=0, blocking=True))
    assert any(d.sync for d in decs_e) and not all(d.sync for d in decs_e)

    graphed = fresh()
    graphed.ctx.step(graphed.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=1)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graphed.ctx.step(graphed.plans[0], 0.05, 0.9, 1e-4, 1.0, first_step=0)
    # the capture itself does not execute: state is still that of step 0
    for t in range(6):
        for k in range(K):
            for x in graphed.d_grads[0][k]:
                x.mul_(scales[t + 1] / scales[t])
        g.replay()
        torch.cuda.synchronize()
        d = graphed.ctx.read_decision()
        assert d.flags == decs_e[t].flags and d.sync == decs_e[t].sync
        assert [x.hex() for x in d.norm_sq] == [x.hex() for x in decs_e[t].norm_sq]
        assert [x.hex() for x in d.delta] == [x.hex() for x in decs_e[t].delta]
    for k in range(K):
        for t in range(len(numel)):
            assert PU.to_host(graphed.d_w[k][t]).tobytes() == PU.to_host(eager.d_w[k][t]).tobytes()
            assert PU.to_host(graphed.d_m[k][t]).tobytes() == PU.to_host(eager.d_m[k][t]).tobytes()
    for t in range(len(numel)):
        assert PU.to_host(graphed.d_glob[t]).tobytes() == PU.to_host(eager.d_glob[t]).tobytes()
    assert graphed.ctx.stats() == eager.ctx.stats()
    del g
    eager.close()
    graphed.close()


# ================================================================= caller-owned streams

def test_two_contexts_on_two_caller_streams_do_not_interfere(B):
    """Everything is ordered on the caller's stream and a context shares nothing with another one: two
    contexts (different K, shapes, precisions) step at the same time on two non-default streams, nothing
    blocks between the enqueues, and each matches the oracle step by step."""
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    numel_a, numel_b = [3_000_001, 70001, 0, 33], [2_000_003, 4096, 5]
    a = PU.LockStep(B, numel_a, 3, delta=0.2, window=5, alpha=0.5, seed=31)
    b = PU.LockStep(B, numel_b, 2, delta=0.1, window=4, alpha=0.5, mixed=True, seed=32)
    r = rng(310)
    a.bind_grads(0, [[(r.standard_normal(n) * 1e-2).astype(np.float32) for n in numel_a] for _ in range(3)])
    b.bind_grads(0, [[W.round_to_bf16_bits((r.standard_normal(n) * 1e-2).astype(np.float32)) for n in numel_b]
                     for _ in range(2)])
    torch.cuda.synchronize()                   # the uploads ran on the default stream
    gs_a = [1.0, 1.0, 2.5, 2.5, 2.5, 0.5, 0.5]
    gs_b = [1.0, 3.0, 3.0, 1.0, 1.0, 1.0, 2.0]
    for t in range(7):
        with torch.cuda.stream(s1):
            a.ctx.step(a.plans[0], 0.05, 0.9, 1e-4, gs_a[t], first_step=int(t == 0))       # not blocking
        with torch.cuda.stream(s2):
            b.ctx.step(b.plans[0], 0.02, 0.8, 0.0, gs_b[t], first_step=int(t == 0))
        s1.synchronize()
        s2.synchronize()
        for ls, (lr, mu, wd), gs in ((a, (0.05, 0.9, 1e-4), gs_a[t]), (b, (0.02, 0.8, 0.0), gs_b[t])):
            dec = ls.ctx.read_decision()
            rec = ls._oracle_track_and_update(0, lr, mu, wd, gs, t == 0, False)
            sync = ls._check_decision(dec, rec)
            if sync:
                ls._oracle_average()
            ls.steps_done += 1
            ls.compare(after_sync=bool(sync))
    for ls in (a, b):
        assert ls.oracle.steps_sync > 0 and ls.oracle.steps_local > 0 and ls.worst_ulp == 0 and ls.forced == 0
        st = ls.ctx.stats()
        assert st["steps_sync"] == ls.oracle.steps_sync and st["steps_local"] == ls.oracle.steps_local
        ls.close()


# ================================================================= fully synchronous step in one pass

@pytest.mark.parametrize("K", [1, 2, 3, 4, 8, 17])
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign,misalign_g", [(0, 0), (1, 1), (2, 3)])
def test_one_pass_synchronous_step_matches_oracle(B, K, mixed, misalign, misalign_g):
    # update + tracking + unconditional aggregation in one kernel; compile-time K, run-time K (3, 17),
    # vector path (equal address phases), peeled heads (1, 1) and the element-wise path (2, 3)
    numel = [70001, 5, 4096, 0, 1023, 255, 257]
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign,
                     misalign_g=misalign_g, seed=81, tuning=dict(nontemporal=K % 2))
    r = rng(810 + K)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot) * (1 + 0.1 * k)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    flagged = 0
    for t in range(7):
        dec, rec = ls.step_bsp([0, 1, 2, 2, 0, 1, 1][t], 0.05, 0.9, [0.0, 1e-4][t % 2], [1.0, 0.7][t % 2],
                               nesterov=(t >= 5))
        flagged += rec.sync
        for tt in range(len(numel)):         # the averaged model is bit-identical to the oracle's
            assert PU.to_host(ls.d_glob[tt]).tobytes() == ls.h_glob[tt].tobytes()
    assert 0 < flagged < 7                   # the tracker still follows its threshold; the aggregation ignores it
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12 and ls.forced == 0
    got = ls.ctx.read_tensor_norms(ls.plans[1])          # per-tensor norms come from this pass's partials
    for k in range(K):
        for t in range(len(numel)):
            assert got[k][t] == pytest.approx(O.norm_sq([ls.h_grads[1][k][t]], 1.0), rel=1e-12, abs=0.0)
    st = ls.ctx.stats()
    assert st["steps_sync"] == ls.oracle.steps_sync and st["steps_local"] == ls.oracle.steps_local
    ls.close()


@pytest.mark.parametrize("mixed", [False, True])
def test_one_pass_synchronous_step_on_momentum_free_plans(B, mixed):
    numel = [70001, 5, 4096, 0, 1023]
    K = 4
    ls = PU.LockStep(B, numel, K, delta=0.0, mixed=mixed, seed=82, momentum_free=True)
    r = rng(820)
    for slot in range(2):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    for t in range(5):
        dec, rec = ls.step_bsp(t % 2, 2.0 * 0.8 ** t, 0.0, [0.0, 1e-4][t % 2], 1.0)
        assert dec.sync == 1
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    ls.close()


@pytest.mark.parametrize("K", [1, 3, 4, 8])
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign,misalign_g", [(0, 0), (1, 1), (2, 3)])
def test_one_pass_synchronous_step_with_adam_matches_oracle(B, K, mixed, misalign, misalign_g):
    numel = [70001, 5, 4096, 0, 1023, 255]
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign,
                     misalign_g=misalign_g, seed=84, tuning=dict(nontemporal=K % 2))
    r = rng(840 + K)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot) * (1 + 0.1 * k)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    ls.enable_adam()
    flagged = 0
    for t in range(6):
        dec, rec = ls.step_bsp_adam([0, 1, 2, 2, 0, 1][t], 1e-3, 0.9, 0.999, 1e-8, [0.0, 1e-2][t % 2], [1.0, 0.7][t % 2])
        flagged += rec.sync
        for tt in range(len(numel)):
            assert PU.to_host(ls.d_glob[tt]).tobytes() == ls.h_glob[tt].tobytes()
    assert 0 < flagged < 6 and ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    ls.close()


def test_adam_step_at_threshold_zero_takes_the_one_pass_kernel_with_identical_results(B):
    numel = [100003, 257, 65536]
    K = 4
    runs = []
    for fused in (True, False):
        ls = PU.LockStep(B, numel, K, delta=0.0, alpha=0.5, window=5, seed=85)
        rr = rng(850)
        for slot in range(2):
            ls.bind_grads(slot, [[(rr.standard_normal(n) * (1 + slot) * 1e-2).astype(np.float32) for n in numel]
                                 for _ in range(K)])
        ls.enable_adam()
        ls.ctx.profile_enable(True, 64)
        decs = [ls.step_adam(t % 2, 1e-3, 0.9, 0.999, 1e-8, 1e-2, 1.0, fused=fused)[0] for t in range(5)]
        launches = [ls.ctx.profile_summary(kind)[0] for kind in range(3)]
        assert launches == ([5, 5, 0] if fused else [10, 5, 5])
        state = [[PU.to_host(x).tobytes() for x in ls.d_w[k] + ls.d_m[k] + ls.d_v[k]] for k in range(K)]
        runs.append((decs, state, [PU.to_host(x).tobytes() for x in ls.d_glob]))
        assert ls.oracle.steps_sync == 5 and ls.worst_ulp == 0
        ls.close()
    (d1, s1, g1), (d2, s2, g2) = runs
    assert s1 == s2 and g1 == g2
    for a, b in zip(d1, d2):
        assert a.sync == b.sync == 1 and [x.hex() for x in a.norm_sq] == [x.hex() for x in b.norm_sq]


@pytest.mark.parametrize("mixed", [False, True])
def test_step_at_threshold_zero_takes_the_one_pass_kernel_with_identical_results(B, mixed):
    """selsync_step under delta = 0 runs the one-pass kernel; the three-call sequence runs the update pass
    and the aggregation pass.  Same tensors bit for bit, and (buffers of a tensor at equal addresses modulo
    1 KiB, as here) the same bits in norms and Delta."""
    numel = [100003, 257, 65536, 4096]
    K = 4
    runs = []
    for fused in (True, False):
        ls = PU.LockStep(B, numel, K, delta=0.0, alpha=0.5, window=5, mixed=mixed, seed=83)
        rr = rng(830)
        for slot in range(3):
            grads = []
            for k in range(K):
                gk = [(rr.standard_normal(n) * (1 + slot) * 1e-2).astype(np.float32) for n in numel]
                grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
            ls.bind_grads(slot, grads)
        ls.ctx.profile_enable(True, 64)
        decs = [ls.step(t % 3, 0.05, 0.9, 1e-4, 1.0, fused=fused)[0] for t in range(6)]
        launches = [ls.ctx.profile_summary(kind)[0] for kind in range(3)]
        # one-pass: 6 launches of the streaming kind, none of the aggregation kind; three calls: 12 and 6
        assert launches == ([6, 6, 0] if fused else [12, 6, 6])
        state = [[PU.to_host(x).tobytes() for x in ls.d_w[k]] + [PU.to_host(x).tobytes() for x in ls.d_m[k]]
                 for k in range(K)]
        runs.append((decs, state, [PU.to_host(x).tobytes() for x in ls.d_glob]))
        assert ls.oracle.steps_sync == 6 and ls.worst_ulp == 0
        ls.close()
    (d1, s1, g1), (d2, s2, g2) = runs
    assert s1 == s2 and g1 == g2
    for a, b in zip(d1, d2):
        assert a.flags == b.flags and a.sync == b.sync == 1
        assert [x.hex() for x in a.norm_sq] == [x.hex() for x in b.norm_sq]
        assert [x.hex() for x in a.delta] == [x.hex() for x in b.delta]


# ================================================================= data partitioning (Sec. III-D)

@pytest.mark.parametrize("D,N", [(100, 4), (103, 4), (5, 8), (0, 3), (1_000_003, 16)])
def test_partition_order_kernel_matches_oracle(B, D, N):
    for n in sorted({0, 1 % N, N - 1}):
        for seldp in (True, False):
            got = B.partition_order_device(D, N, n, seldp).cpu().tolist()
            want = O.seldp_order(D, N, n) if seldp else O.defdp_order(D, N, n)
            assert got == want


# ================================================================= variant: Adam local update

@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1])
def test_adam_variant_matches_oracle(B, mixed, misalign):
    numel = [70001, 5, 4096, 0, 1023]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=21,
                     tuning=dict(nontemporal=int(misalign == 0)))
    r = rng(140)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    with pytest.raises(B.SelSyncError) as e:                 # Adam needs its second-moment buffers
        ls.ctx.local_step_adam(ls.plans[0], 1e-3)
    assert e.value.status == B.SELSYNC_ERR_STATE
    ls.enable_adam()
    syncs = 0
    for t in range(9):
        dec, rec = ls.step_adam([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 1e-3, 0.9, 0.999, 1e-8, [0.0, 1e-2][t % 2],
                                [1.0, 0.7][t % 2], fused=(t % 3 != 1))
        syncs += rec.sync
    assert 0 < syncs < 9
    assert ls.worst_ulp == 0          # same rounding sequence, correctly rounded divide / sqrt on both sides
    ls.close()


def test_adam_bind_validation(B):
    K = 2
    ctx = B.SelSync(K, 0.3)
    mk = lambda n: torch.zeros(n, dtype=torch.float32, device="cuda")
    g, p, m, glob = [[mk(100)] for _ in range(K)], [[mk(100)] for _ in range(K)], [[mk(100)] for _ in range(K)], [mk(100)]
    plan = ctx.plan(g, p, m, glob)
    def status(fn):
        with pytest.raises(B.SelSyncError) as e:
            fn()
        return e.value.status
    assert status(lambda: ctx.bind_second_moment(plan, [[mk(99)], [mk(100)]])) == B.SELSYNC_ERR_SHAPE_MISMATCH
    assert status(lambda: ctx.bind_second_moment(plan, m)) == B.SELSYNC_ERR_INVALID_ARG          # overlaps momenta
    v = [[mk(100)] for _ in range(K)]
    assert status(lambda: ctx.bind_second_moment(plan, [v[0], v[0]])) == B.SELSYNC_ERR_INVALID_ARG
    ctx.bind_second_moment(plan, v)
    ctx.bind_second_moment(plan, v)                                                              # re-binding is fine
    assert status(lambda: ctx.local_step_adam(plan, 1e-3, beta1=1.0)) == B.SELSYNC_ERR_INVALID_ARG
    ctx.local_step_adam(plan, 1e-3)
    agg_only = ctx.plan(None, p, None, glob)
    assert status(lambda: ctx.bind_second_moment(agg_only, v)) == B.SELSYNC_ERR_STATE
    ctx.close()


# ================================================================= variant: gradient aggregation

@pytest.mark.parametrize("K", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1])
def test_gradient_aggregation_matches_oracle(B, K, mixed, misalign):
    numel = [70001, 5, 4096, 0, 1023]
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=19,
                     tuning=dict(nontemporal=K % 2))
    r = rng(110 + K)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    # let the replicas drift apart first so that "replicas stay apart" is visible
    for k in range(K):
        for t, n in enumerate(numel):
            ls.h_w[k][t] += np.float32(1e-3 * k)
            ls.d_w[k][t].copy_(torch.from_numpy(ls.h_w[k][t]))
            if mixed:
                ls.h_c[k][t][...] = W.round_to_bf16_bits(ls.h_w[k][t])
                ls.d_c[k][t].copy_(PU.to_dev(ls.h_c[k][t]))
    syncs = 0
    for t in range(9):
        dec, rec = ls.step_ga([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 0.05, 0.9, 1e-4, [1.0, 0.7][t % 2], fused=(t % 3 != 1))
        syncs += rec.sync
    assert syncs > 0 and syncs < 9 and ls.worst_ulp == 0
    if K > 1:       # Sec. III-C: after gradient aggregation the workers' models are still different
        assert PU.to_host(ls.d_w[0][0]).tobytes() != PU.to_host(ls.d_w[K - 1][0]).tobytes()
    ls.close()


def test_gradient_aggregation_always_mode_and_bsp_equivalence(B):
    # from identical replicas, aggregating every step keeps all workers bit-identical (BSP with GA)
    numel = [33333, 100]
    K = 4
    ls = PU.LockStep(B, numel, K, delta=float("inf"), seed=20)
    for slot in range(2):
        ls.bind_grads(slot, [[rng(130 + 10 * slot + k).standard_normal(n).astype(np.float32) for n in numel]
                             for k in range(K)])
    for t in range(4):
        ls.ctx.ga_update(ls.plans[t % 2], 0.1, 0.9, 5e-4, 1.0, first_step=int(t == 0), always=True)
        O.ga_update(ls.h_grads[t % 2], ls.h_w, ls.h_m, 0.1, 0.9, 5e-4, 1.0, t == 0, True)
        ls.compare()
        for k in range(1, K):
            assert PU.to_host(ls.d_w[k][0]).tobytes() == PU.to_host(ls.d_w[0][0]).tobytes()
    ls.close()


@pytest.mark.parametrize("K", [2, 3, 4, 8])
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1])
def test_gradient_aggregation_on_momentum_free_plans(B, K, mixed, misalign):
    # Sec. III-C with the momentum-free SGD of the Transformer recipe: no buffer is bound, read or written
    numel = [70001, 5, 4096, 0, 1023]
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=24,
                     momentum_free=True, tuning=dict(nontemporal=K % 2, ga_chunk_elems=[0, 256][misalign]))
    r = rng(240 + K)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    for k in range(K):                          # replicas start apart: they must stay apart
        for t, n in enumerate(numel):
            ls.h_w[k][t] += np.float32(1e-3 * k)
            ls.d_w[k][t].copy_(torch.from_numpy(ls.h_w[k][t]))
            if mixed:
                ls.h_c[k][t][...] = W.round_to_bf16_bits(ls.h_w[k][t])
                ls.d_c[k][t].copy_(PU.to_dev(ls.h_c[k][t]))
    syncs = 0
    for t in range(9):
        dec, rec = ls.step_ga([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 2.0 * 0.8 ** t, 0.0, [0.0, 1e-4][t % 2], [1.0, 0.7][t % 2],
                              fused=(t % 3 != 1))
        syncs += rec.sync
    assert 0 < syncs < 9 and ls.worst_ulp == 0
    assert PU.to_host(ls.d_w[0][0]).tobytes() != PU.to_host(ls.d_w[K - 1][0]).tobytes()
    # always-mode on the bandwidth-shaped table
    ls.ctx.ga_update(ls.plans[0], 0.1, 0.0, 1e-4, 0.5, always=True)
    O.ga_update(ls.h_grads[0], ls.h_w, None, 0.1, 0.0, 1e-4, 0.5, False, True, ls.h_c)
    ls.compare()
    ls.close()


@pytest.mark.parametrize("K", [1, 3, 4, 8])
@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 1])
def test_gradient_aggregation_with_adam_matches_oracle(B, K, mixed, misalign):
    # every worker feeds the mean gradient to its own Adam state on "sync", its own gradient on "local"
    numel = [70001, 5, 4096, 0, 1023]
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=25,
                     tuning=dict(nontemporal=int(misalign == 0), ga_chunk_elems=[0, 512][K % 2]))
    r = rng(250 + K)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    for k in range(K):
        for t, n in enumerate(numel):
            ls.h_w[k][t] += np.float32(1e-3 * k)
            ls.d_w[k][t].copy_(torch.from_numpy(ls.h_w[k][t]))
            if mixed:
                ls.h_c[k][t][...] = W.round_to_bf16_bits(ls.h_w[k][t])
                ls.d_c[k][t].copy_(PU.to_dev(ls.h_c[k][t]))
    with pytest.raises(B.SelSyncError) as e:                 # needs its second-moment buffers
        ls.ctx.ga_update_adam(ls.plans[0], 1e-3)
    assert e.value.status == B.SELSYNC_ERR_STATE
    ls.enable_adam()
    syncs = 0
    for t in range(9):
        dec, rec = ls.step_ga_adam([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 1e-3, 0.9, 0.999, 1e-8, [0.0, 1e-2][t % 2],
                                   [1.0, 0.7][t % 2], fused=(t % 3 != 1))
        syncs += rec.sync
    assert 0 < syncs < 9 and ls.worst_ulp == 0
    if K > 1:
        assert PU.to_host(ls.d_w[0][0]).tobytes() != PU.to_host(ls.d_w[K - 1][0]).tobytes()
    # always-mode on the bandwidth-shaped table
    t = ls.steps_done + 1
    ls.ctx.ga_update_adam(ls.plans[1], 1e-3, 0.9, 0.999, 1e-8, 0.0, 0.5, step=t, always=True)
    O.ga_update_adam(ls.h_grads[1], ls.h_w, ls.h_m, ls.h_v, 1e-3, 0.9, 0.999, 1e-8, 0.0, t, 0.5, True, ls.h_c)
    ls.compare()
    ls.close()


# ================================================================= many workers

@pytest.mark.parametrize("K", [17, 40, 130])
@pytest.mark.parametrize("mixed", [False, True])
def test_more_workers_than_one_tracker_round(B, K, mixed):
    # the tracker workgroup handles 16 workers per round; the K-way kernels take the run-time-K path
    numel = [3001, 64, 0, 7]
    ls = PU.LockStep(B, numel, K, delta=0.2, window=6, mixed=mixed, seed=50 + K)
    r = rng(180 + K)
    for slot in range(2):
        grads = []
        for k in range(K):
            scale = 1e-2 * (1 + 4 * slot) * (1.0 + 0.01 * k)
            gk = [(r.standard_normal(n) * scale).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    syncs = 0
    for t in range(6):
        dec, rec = ls.step([0, 0, 1, 1, 0, 1][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
        syncs += rec.sync
        assert len(dec.norm_sq) == K and dec.flags == rec.flags
    for t in range(3):
        dec, rec = ls.step_ga([1, 0, 1][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
        syncs += rec.sync
    assert 0 < syncs < 9 and ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    st = ls.ctx.stats()
    assert st["steps_sync"] == ls.oracle.steps_sync and st["steps_local"] == ls.oracle.steps_local
    ls.close()


def test_the_largest_worker_count_a_context_accepts(B):
    # 1024 workers is the limit of selsync_create: 64 tracker rounds, run-time K in every K-way kernel
    K = 1024
    with pytest.raises(B.SelSyncError):
        B.SelSync(K + 1, 0.2)
    numel = [300, 0, 5]
    ls = PU.LockStep(B, numel, K, delta=0.2, window=4, seed=61)
    r = rng(190)
    for slot in range(2):
        ls.bind_grads(slot, [[(r.standard_normal(n) * 1e-2 * (1 + 3 * slot) * (1.0 + 0.001 * k)).astype(np.float32)
                              for n in numel] for k in range(K)])
    syncs = 0
    for t in range(4):
        dec, rec = ls.step([0, 0, 1, 1][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
        syncs += rec.sync
        assert len(dec.norm_sq) == K and dec.flags == rec.flags
    dec, rec = ls.step_ga(0, 0.05, 0.9, 1e-4, 1.0)
    dec, rec = ls.step_bsp(1, 0.05, 0.9, 1e-4, 1.0)
    assert 0 < syncs < 4 and ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    ls.close()


# ================================================================= tensors anywhere in an arena

@pytest.mark.parametrize("off_w,off_g", [(37, 37), (37, 41), (100, 4), (255, 255), (260, 0), (64, 192), (129, 2)])
@pytest.mark.parametrize("mixed", [False, True])
def test_tensors_at_arbitrary_offsets_inside_larger_buffers(B, off_w, off_g, mixed):
    # pieces are cut where addresses cross multiples of the chunk size, whatever the tensor's start address is;
    # parameters/momenta and gradients may sit at different offsets (equal or different vector phase)
    numel = [70001, 5, 4096, 0, 1023, 255, 257]
    K = 2
    for tuning in (None, dict(chunk_elems=1024, agg_chunk_elems=512, ga_chunk_elems=256)):
        ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=off_w, misalign_g=off_g,
                         seed=41, tuning=tuning)
        r = rng(170)
        for slot in range(2):
            grads = []
            for k in range(K):
                gk = [(r.standard_normal(n) * 1e-2 * (1 + 3 * slot)).astype(np.float32) for n in numel]
                grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
            ls.bind_grads(slot, grads)
        syncs = 0
        for t in range(6):
            dec, rec = ls.step([0, 1, 1, 0, 1, 0][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
            syncs += rec.sync
        for t in range(3):
            dec, rec = ls.step_ga([1, 0, 1][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0))
            syncs += rec.sync
        assert 0 < syncs < 9 and ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
        got = ls.ctx.read_tensor_norms(ls.plans[1])
        for k in range(K):
            for t in range(len(numel)):
                assert got[k][t] == pytest.approx(O.norm_sq([ls.h_grads[1][k][t]], 1.0), rel=1e-12, abs=0.0)
        ls.close()


# ================================================================= seeded random configurations

@pytest.mark.parametrize("seed", list(range(96)))
def test_random_configuration_matches_oracle(B, seed):
    """Random tensor lists, placements, worker counts and launch shapes; fused, three-call and
    gradient-aggregation steps in one run, everything compared with the oracle."""
    r = rng(1000 + seed + int(os.environ.get("SELSYNC_TEST_SEED_OFFSET", "0")))     # offset: further cases on request
    sizes = [0, 1, 2, 3, 5, 63, 64, 255, 256, 257, 511, 1000, 1024, 4099, 8192, 70001]
    K = int(r.integers(1, 7))
    T = int(r.integers(1, 9))
    numel = [int(r.choice(sizes)) for _ in range(T)]
    if sum(numel) == 0:
        numel[0] = 777
    mixed = bool(r.integers(0, 2))
    chunk = int(r.choice([256, 512, 1024, 4096]))
    tuning = dict(chunk_elems=chunk, nontemporal=int(r.integers(0, 2)),
                  agg_chunk_elems=int(r.choice([0, 256, 1024, 4096])), ga_chunk_elems=int(r.choice([0, 256, 1024])))
    off = lambda: int(r.choice([0, 0, 1, 2, 3, 4, 17, 64, 100, 255, 256, 300]))
    momentum_free = bool(r.integers(0, 4) == 0)
    ls = PU.LockStep(B, numel, K, delta=float(r.choice([0.0, 0.1, 0.3])), window=int(r.choice([1, 3, 25])),
                     alpha=float(r.choice([-1.0, 0.5, 1.0])), mixed=mixed, misalign=off(), misalign_g=off(),
                     misalign_m=off(), misalign_glob=off(), seed=seed, tuning=tuning, momentum_free=momentum_free)
    for slot in range(2):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 3 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    mu = 0.0 if momentum_free else float(r.choice([0.0, 0.9]))
    nesterov = bool(mu > 0 and r.integers(0, 2))
    for t in range(6):
        ls.step(int(r.integers(0, 2)), 0.05, mu, float(r.choice([0.0, 1e-4])), float(r.choice([1.0, 0.5])),
                fused=bool(r.integers(0, 2)), nesterov=nesterov)
    for t in range(3):
        ls.step_ga(int(r.integers(0, 2)), 0.05, mu, 1e-4, 1.0, fused=bool(r.integers(0, 2)), nesterov=nesterov)
    ls.step_bsp(int(r.integers(0, 2)), 0.05, mu, 1e-4, 0.5, nesterov=nesterov)
    if not momentum_free:
        if r.integers(0, 2):
            ls.enable_adam()
            ls.steps_done = 0                      # Adam's bias correction counts its own steps from 1
            for t in range(3):
                ls.step_adam(int(r.integers(0, 2)), 1e-3, 0.9, 0.999, 1e-8, float(r.choice([0.0, 1e-4])), 1.0,
                             fused=bool(r.integers(0, 2)))
            for t in range(2):
                ls.step_ga_adam(int(r.integers(0, 2)), 1e-3, 0.9, 0.999, 1e-8, float(r.choice([0.0, 1e-4])), 1.0,
                                fused=bool(r.integers(0, 2)))
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    st = ls.ctx.stats()
    assert st["steps_sync"] == ls.oracle.steps_sync and st["steps_local"] == ls.oracle.steps_local
    ls.close()


# ================================================================= variants: momentum-free SGD, Nesterov momentum

@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 3])
@pytest.mark.parametrize("tuning", [None, dict(chunk_elems=1024)])
def test_momentum_free_sgd_matches_oracle(B, mixed, misalign, tuning):
    # plain SGD of the Transformer recipe (Sec. IV-A): plans without momentum buffers
    numel = [70001, 5, 4096, 0, 1023]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=31,
                     momentum_free=True, tuning=tuning)
    r = rng(140)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    syncs = 0
    for t in range(9):
        dec, rec = ls.step([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 2.0 * 0.8 ** t, 0.0, [0.0, 1e-4][t % 2], [1.0, 0.7][t % 2],
                           fused=(t % 3 != 1))
        syncs += rec.sync
    assert 0 < syncs < 9 and ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-12
    ls.close()


def test_momentum_free_plan_rejects_momentum_and_adam(B):
    K = 2
    ctx = B.SelSync(K, 0.3)
    mk = lambda n: torch.zeros(n, dtype=torch.float32, device="cuda")
    g, p, glob = [[mk(100)] for _ in range(K)], [[mk(100)] for _ in range(K)], [mk(100)]
    plan = ctx.plan(g, p, None, glob)

    def status(fn):
        with pytest.raises(B.SelSyncError) as e:
            fn()
        return e.value.status

    ctx.local_step(plan, 0.1, 0.0)
    assert status(lambda: ctx.local_step(plan, 0.1, 0.9)) == B.SELSYNC_ERR_INVALID_ARG
    assert status(lambda: ctx.step(plan, 0.1, 0.0, nesterov=True)) == B.SELSYNC_ERR_INVALID_ARG
    ctx.ga_update(plan, 0.1, 0.0)                       # gradient aggregation works without momentum buffers ...
    ctx.step_ga(plan, 0.1, 0.0)
    assert status(lambda: ctx.ga_update(plan, 0.1, 0.9)) == B.SELSYNC_ERR_INVALID_ARG      # ... with momentum 0
    assert status(lambda: ctx.step_ga(plan, 0.1, 0.9)) == B.SELSYNC_ERR_INVALID_ARG
    assert status(lambda: ctx.bind_second_moment(plan, [[mk(100)] for _ in range(K)])) == B.SELSYNC_ERR_STATE
    assert status(lambda: ctx.ga_update_adam(plan, 1e-3)) == B.SELSYNC_ERR_STATE
    assert status(lambda: ctx.step_ga_adam(plan, 1e-3)) == B.SELSYNC_ERR_STATE
    # momenta without gradients make no sense
    assert status(lambda: ctx.plan(None, p, [[mk(100)] for _ in range(K)], glob)) == B.SELSYNC_ERR_INVALID_ARG
    # Nesterov needs momentum > 0 on an ordinary plan too
    full = ctx.plan(g, p, [[mk(100)] for _ in range(K)], glob)
    assert status(lambda: ctx.local_step(full, 0.1, 0.0, nesterov=True)) == B.SELSYNC_ERR_INVALID_ARG
    sgd = B.selsync_sgd(0.1, 0.9, 0.0, 1.0, 0, 2)
    assert B.selsync_local_step(ctx._h, full._h, ctypes.byref(sgd), None) == B.SELSYNC_ERR_INVALID_ARG
    ctx.close()


@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("misalign", [0, 2])
def test_nesterov_momentum_matches_oracle(B, mixed, misalign):
    numel = [70001, 5, 4096, 0, 1023]
    K = 3
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, misalign=misalign, seed=32)
    r = rng(150)
    for slot in range(3):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 2 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    syncs = 0
    for t in range(9):
        dec, rec = ls.step([0, 1, 2, 2, 0, 1, 1, 2, 0][t], 0.05, 0.9, 1e-4, [1.0, 0.7][t % 2], fused=(t % 3 != 1),
                           nesterov=True)
        syncs += rec.sync
    assert 0 < syncs < 9 and ls.worst_ulp == 0
    ls.close()


@pytest.mark.parametrize("mixed", [False, True])
def test_nesterov_under_gradient_aggregation_matches_oracle(B, mixed):
    numel = [33333, 7, 2048]
    K = 4
    ls = PU.LockStep(B, numel, K, delta=0.15, window=5, alpha=0.5, mixed=mixed, seed=33)
    r = rng(160)
    for slot in range(2):
        grads = []
        for k in range(K):
            gk = [(r.standard_normal(n) * 1e-2 * (1 + 3 * slot)).astype(np.float32) for n in numel]
            grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
        ls.bind_grads(slot, grads)
    syncs = 0
    for t in range(6):
        dec, rec = ls.step_ga([0, 1, 1, 0, 1, 0][t], 0.05, 0.9, 1e-4, 1.0, fused=(t % 2 == 0), nesterov=True)
        syncs += rec.sync
    assert 0 < syncs < 6 and ls.worst_ulp == 0
    ls.close()


# ================================================================= the five workloads, lock step

@pytest.mark.parametrize("name,shrink,steps,compare_every,min_syncs", [
    ("c1", 1, 50, 1, 1),         # full size, every tensor after every step
    ("c2", 4, 200, 20, 1),       # stated step counts; channel widths divided by 4 so that the oracle
    ("c3", 4, 200, 40, 0),       # finishes in seconds (the full-size runs are in test_gpu_fullsize.py)
    ("c4", 4, 200, 25, 7),
    ("c5", 4, 500, 50, 0),       # constant gradient scale: the stated schedule never crosses delta = 0.1
])
def test_workload_lockstep(B, name, shrink, steps, compare_every, min_syncs):
    """The five configurations over ALL their steps: decisions, norms and Delta compared every step,
    tensors every `compare_every` steps, at every synchronising step and at the end."""
    wl = W.get(name, shrink=shrink)
    assert wl.steps == steps
    ls = PU.run_workload(B, wl, steps=steps, compare_every=compare_every, oracle_threads=wl.num_workers,
                         progress_every=100)
    print("%s: steps=%d sync=%d lssr=%.3f min|Delta-delta|=%.3g worst norm rel=%.2g worst ulp=%d forced=%d" % (
        wl.name, ls.steps_done, ls.oracle.steps_sync, ls.oracle.lssr, ls.min_margin, ls.worst_norm_rel,
        ls.worst_ulp, ls.forced))
    assert ls.steps_done == steps
    assert ls.min_margin > 1e-3, "seed puts a decision too close to the threshold for a meaningful run"
    assert ls.forced == 0 and ls.worst_ulp == 0
    assert ls.oracle.steps_sync >= min_syncs          # the schedule contains real synchronisations
    ls.close()


def test_mixed_precision_workload_with_sync_steps(B):
    # the stated C5 schedule is constant (never syncs); add spikes so the bf16 aggregation path runs in a workload
    wl = W.get("c5", shrink=8)
    wl.sigma = lambda t: 4.0 if t in (5, 12) else 1.0
    ls = PU.run_workload(B, wl, steps=16, compare_every=1)
    assert ls.oracle.steps_sync >= 2
    ls.close()


# ================================================================= error paths through the C ABI

def _lists(B, tensors_per_worker):
    arr, keep = B._marshal_lists(tensors_per_worker)
    return arr, keep


def test_plan_validation_errors(B):
    K = 2
    ctx = B.SelSync(K, 0.3)
    mk = lambda n, dt=torch.float32: torch.zeros(n, dtype=dt, device="cuda")
    good = lambda: [[mk(100), mk(7)] for _ in range(K)]
    g, p, m, glob = good(), good(), good(), [mk(100), mk(7)]
    ctx.plan(g, p, m, glob).destroy()

    def status(fn):
        with pytest.raises(B.SelSyncError) as e:
            fn()
        return e.value.status

    # shape mismatch: numel and tensor count
    bad = good(); bad[1][1] = mk(8)
    assert status(lambda: ctx.plan(bad, p, m, glob)) == B.SELSYNC_ERR_SHAPE_MISMATCH
    bad = good(); bad[1] = bad[1][:1]
    assert status(lambda: ctx.plan(g, p, bad, glob)) == B.SELSYNC_ERR_SHAPE_MISMATCH
    # dtype: bf16 grads without master, fp32 momenta required
    bad = [[mk(100, torch.bfloat16), mk(7, torch.bfloat16)] for _ in range(K)]
    assert status(lambda: ctx.plan(bad, p, m, glob)) == B.SELSYNC_ERR_DTYPE
    assert status(lambda: ctx.plan(g, p, bad, glob)) == B.SELSYNC_ERR_DTYPE
    # mixed mode needs both master and global_lowp
    assert status(lambda: ctx.plan(bad, bad, m, glob, master=p)) == B.SELSYNC_ERR_INVALID_ARG
    # overlapping written buffers
    assert status(lambda: ctx.plan(g, [p[0], p[0]], m, glob)) == B.SELSYNC_ERR_INVALID_ARG
    assert status(lambda: ctx.plan(g, p, p, glob)) == B.SELSYNC_ERR_INVALID_ARG
    assert status(lambda: ctx.plan(p, p, m, glob)) == B.SELSYNC_ERR_INVALID_ARG
    # the same read-only gradient for every worker is allowed
    ctx.plan([g[0], g[0]], p, m, glob).destroy()
    # host memory is rejected
    host = torch.zeros(100)
    descs = (B.selsync_tensor * 2)()
    descs[0].data, descs[0].numel, descs[0].dtype = host.data_ptr(), 100, B.SELSYNC_F32
    descs[1].data, descs[1].numel, descs[1].dtype = g[0][1].data_ptr(), 7, B.SELSYNC_F32
    ga, keep1 = B._marshal_lists(g)
    pa, keep2 = B._marshal_lists(p)
    ma, keep3 = B._marshal_lists(m)
    gl, keep4 = B._marshal_lists([glob])
    ga[0].tensors = descs
    h = ctypes.c_void_p()
    rc = B.selsync_plan_create(ctx._h, ga, pa, ma, None, gl, None, ctypes.byref(h))
    assert rc == B.SELSYNC_ERR_NOT_DEVICE_MEM and h.value is None
    assert b"not" in B.selsync_last_error(ctx._h)
    # NULL data with numel > 0
    descs[0].data = None
    rc = B.selsync_plan_create(ctx._h, ga, pa, ma, None, gl, None, ctypes.byref(h))
    assert rc == B.SELSYNC_ERR_INVALID_ARG
    # aggregate-only plan: tracking / update are state errors
    plan = ctx.plan(None, p, None, glob)
    assert status(lambda: ctx.track_grad_change(plan)) == B.SELSYNC_ERR_STATE
    assert status(lambda: ctx.local_step(plan, 0.1)) == B.SELSYNC_ERR_STATE
    ctx.aggregate_params(plan, always=True)
    assert B.selsync_aggregate_params(ctx._h, plan._h, 5, None) == B.SELSYNC_ERR_INVALID_ARG
    # destroying a context with live plans is refused
    assert B.selsync_destroy(ctx._h) == B.SELSYNC_ERR_STATE
    ctx.close()


def test_empty_model_and_single_worker(B):
    ctx = B.SelSync(1, 0.3)
    plan = ctx.plan([[]], [[]], [[]], [])
    dec = ctx.step(plan, 0.1, 0.9, 0.0, blocking=True)
    assert dec.norm_sq == [0.0] and dec.sync == 0
    assert plan.info() == {"num_tensors": 0, "num_params": 0, "update_chunks": 0, "aggregate_chunks": 0}
    ctx.close()
    # K = 1: aggregation copies the single replica into the global model
    ls = PU.LockStep(B, [5000, 3], 1, delta=0.0, seed=15)
    ls.bind_grads(0, [[rng(90).standard_normal(n).astype(np.float32) for n in [5000, 3]]])
    ls.step(0, 0.1, 0.9, 1e-4)
    for t in range(2):
        assert PU.to_host(ls.d_glob[t]).tobytes() == PU.to_host(ls.d_w[0][t]).tobytes()
    ls.close()


def test_profile_counters_report_launches(B):
    ls = PU.LockStep(B, [300000], 2, delta=0.3, seed=16)      # (under delta = 0 a step is one kernel, not three)
    ls.bind_grads(0, [[rng(95 + k).standard_normal(300000).astype(np.float32)] for k in range(2)])
    ls.ctx.profile_enable(True, 16)
    for _ in range(4):
        ls.ctx.step(ls.plans[0], 0.1, 0.9, 0.0)
    for kind in range(3):
        count, ms = ls.ctx.profile_summary(kind)
        assert count == 4 and ms > 0.0
    ls.ctx.profile_enable(False)
    ls.close()
