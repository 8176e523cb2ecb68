"""Full-size parity in the launch configuration bench.py times (library defaults): the VGG11-shaped
workload (132,863,336 fp32 parameters, K = 4) and the three other stated configurations at their stated
sizes, worker counts and step counts, compared with the CPU oracle element by element.

The whole-schedule tests take one to two minutes each, nearly all of it in the oracle: they print a
progress line past pytest's capture every few dozen steps, so that a watcher sees the run is alive."""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_2307_07950_amd import workloads as W                 # noqa: E402
from tests import parity_util as PU                             # noqa: E402


@pytest.fixture
def progress(capsys):
    def emit(line):
        with capsys.disabled():
            print(line, flush=True)
    return emit


def test_vgg11_like_full_size_three_steps_with_sync():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding as B
    t0 = time.time()
    wl = W.get("c4")
    assert wl.num_params == 132_863_336 and wl.num_workers == 4
    K = wl.num_workers
    ls = PU.LockStep(B, wl.numels, K, wl.delta, wl.window, -1.0, False, init_params=W.initial_params(wl))
    ls.bind_grads(0, [W.unit_grads(wl, k, 0) for k in range(K)])
    info = ls.plans[0].info()
    assert info["num_params"] == wl.num_params and info["update_chunks"] > 1_000_000   # segment level in use
    print("setup %.1fs" % (time.time() - t0), flush=True)
    sig = [1e-3, 1e-3, 4e-3]                      # the workload's 4x spike, moved to step 2
    for t in range(3):
        dec, rec = ls.step(0, wl.lr, wl.momentum, wl.weight_decay, sig[t], fused=True, compare_tensors=False)
        print("step %d sync=%d norm rel err %.2g (%.1fs)" % (t, dec.sync, ls.worst_norm_rel, time.time() - t0),
              flush=True)
        assert dec.sync == rec.sync == (1 if t == 2 else 0)
    # the last step synchronised and was compared in full by the runner (params, momenta, global)
    assert ls.worst_norm_rel < 1e-10      # bar is 1e-5; the sequential fp64 oracle sum itself drifts ~1e-12 here
    assert ls.worst_ulp == 0
    st = ls.ctx.stats()
    assert st["steps_sync"] == 1 and st["steps_local"] == 2
    ls.close()


def test_vgg11_like_full_size_all_200_steps(progress):
    """The 133M-parameter configuration exactly as stated -- full size, K = 4, all 200 steps, library
    defaults (the launch configuration bench.py times): decisions, norms and Delta compared with the
    oracle after every step, every tensor of every replica at each synchronising step and at the end."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding as B
    wl = W.get("c4")
    assert (wl.num_params, wl.num_workers, wl.steps) == (132_863_336, 4, 200)
    ls = PU.run_workload(B, wl, compare_every=0, oracle_threads=16, progress_every=50, progress=progress)
    print("%s: steps=%d sync=%d lssr=%.3f min|Delta-delta|=%.3g worst norm rel=%.2g worst ulp=%d forced=%d" % (
        wl.name, ls.steps_done, ls.oracle.steps_sync, ls.oracle.lssr, ls.min_margin, ls.worst_norm_rel,
        ls.worst_ulp, ls.forced), flush=True)
    assert ls.steps_done == 200 and ls.oracle.steps_sync >= 7
    assert ls.forced == 0 and ls.min_margin > 1e-3
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-10
    ls.close()


@pytest.mark.parametrize("name,params,workers,steps", [("c2", 44_541_480, 8, 200), ("c3", 61_100_840, 8, 200),
                                                       ("c5", 61_212_158, 8, 500)])
def test_other_workloads_full_size_all_steps(name, params, workers, steps, progress):
    """The ResNet-, AlexNet- and Transformer-shaped configurations exactly as stated: full size, K = 8, all 200 / 200 /
    500 steps, library defaults.  Decisions, norms and Delta are compared with the oracle after every step, every tensor
    at each synchronising step and at the end (the AlexNet- and Transformer-shaped schedules have a constant gradient
    scale and never reach their thresholds: for them the chain of 200 / 500 local updates is what is checked)."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding as B
    wl = W.get(name)
    assert (wl.num_params, wl.num_workers, wl.steps) == (params, workers, steps)
    ls = PU.run_workload(B, wl, compare_every=0, oracle_threads=16, progress_every=100, progress=progress)
    print("%s: steps=%d sync=%d lssr=%.3f min|Delta-delta|=%.3g worst norm rel=%.2g worst ulp=%d forced=%d" % (
        wl.name, ls.steps_done, ls.oracle.steps_sync, ls.oracle.lssr, ls.min_margin, ls.worst_norm_rel,
        ls.worst_ulp, ls.forced), flush=True)
    assert ls.steps_done == steps and ls.forced == 0 and ls.min_margin > 1e-3
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-9
    if name == "c2":
        assert ls.oracle.steps_sync >= 1
    ls.close()


def test_vgg11_like_full_size_fully_synchronous_steps():
    """The 133M-parameter configuration at full size under a threshold of 0 (BSP): selsync_step takes the
    one-pass kernel; three steps, every tensor of every replica compared with the oracle after the last."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding as B
    wl = W.get("c4")
    wl.delta = 0.0
    ls = PU.run_workload(B, wl, steps=3, compare_every=0, oracle_threads=wl.num_workers, pool=1)
    assert ls.oracle.steps_sync == 3 and ls.forced == 0
    assert ls.worst_ulp == 0 and ls.worst_norm_rel < 1e-10
    for t in range(len(wl.numels)):
        assert PU.to_host(ls.d_glob[t]).tobytes() == ls.h_glob[t].tobytes()
    ls.close()


@pytest.mark.parametrize("name,params,tensors,workers", [("c2", 44_541_480, 314, 8), ("c3", 61_100_840, 16, 8),
                                                         ("c5", 61_212_158, 186, 8)])
def test_other_workloads_full_size_local_step_then_sync(name, params, tensors, workers):
    """The ResNet-, AlexNet- and Transformer-shaped workloads at full size (the last one in bf16 mixed
    precision), library defaults: one local step, then a step whose 4x gradient spike synchronises;
    every tensor of every replica is compared with the oracle after both."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding as B
    t0 = time.time()
    wl = W.get(name)
    assert (wl.num_params, wl.num_tensors, wl.num_workers) == (params, tensors, workers)
    K = wl.num_workers
    ls = PU.LockStep(B, wl.numels, K, wl.delta, wl.window, -1.0, wl.mixed_bf16, init_params=W.initial_params(wl))
    ls.bind_grads(0, [W.unit_grads(wl, k, 0) for k in range(K)])
    print("%s setup %.1fs" % (name, time.time() - t0), flush=True)
    base = float(np.float32(wl.sigma(0)))
    for t, sig in enumerate([base, 4.0 * base]):
        dec, rec = ls.step(0, wl.lr, wl.momentum, wl.weight_decay, sig, fused=True, compare_tensors=True)
        print("%s step %d sync=%d norm rel err %.2g ulp %d (%.1fs)" % (name, t, dec.sync, ls.worst_norm_rel,
                                                                     ls.worst_ulp, time.time() - t0), flush=True)
        assert dec.sync == rec.sync == t
    # bar: 1e-5.  The oracle adds 61 M squares in index order; on the bf16 workload with its 100x spread of
    # per-tensor scales that in-order fp64 sum is itself 1.5e-10 away from a long-double reference (the
    # kernel's tree-shaped sum is the closer one), so "agrees to 1e-9" is what can be asked of the pair.
    assert ls.worst_norm_rel < 1e-9 and ls.worst_ulp == 0
    ls.close()


def test_tensor_beyond_2_to_31_elements_uses_64_bit_offsets():
    """One tensor of 2^31 + 12345 elements (8.6 GB per buffer): every chunk offset past 2^31 must be
    addressed correctly.  Checked through properties that hold at any size: a constant gradient c
    gives ||g||^2 = n c^2 exactly, and a constant state stays constant with the value the oracle
    computes for a single element."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    free, _ = torch.cuda.mem_get_info()
    n = (1 << 31) + 12345
    if free < 5 * 4 * n:
        pytest.skip("not enough free HBM for a 2^31-element case")
    from oracle import selsync_oracle as O
    from paper_2307_07950_amd import binding as B
    import numpy as np
    g = torch.full((n,), 0.5, dtype=torch.float32, device="cuda")
    w = torch.full((n,), 1.25, dtype=torch.float32, device="cuda")
    m = torch.full((n,), -0.75, dtype=torch.float32, device="cuda")
    glob = torch.zeros(n, dtype=torch.float32, device="cuda")
    ctx = B.SelSync(1, 0.0)                               # delta 0: the step also aggregates (copies w to global)
    plan = ctx.plan([[g]], [[w]], [[m]], [glob])
    assert plan.info()["update_chunks"] == -(-n // 256)
    dec = ctx.step(plan, 0.1, 0.9, 5e-4, 2.0, first_step=0, blocking=True)
    assert dec.norm_sq == [float(n)]                      # (2*0.5)^2 * n, exact in fp64
    hw, hm, hg = np.array([1.25], np.float32), np.array([-0.75], np.float32), np.array([0.5], np.float32)
    O.sgd_update([hw], [hm], [hg], 0.1, 0.9, 5e-4, 2.0, False)
    for t, want in ((w, hw[0]), (m, hm[0]), (glob, hw[0])):
        assert float(t.min()) == float(want) and float(t.max()) == float(want)
    assert float(w[-1]) == float(hw[0]) and float(w[(1 << 31) + 5]) == float(hw[0])
    assert dec.sync == 1
    ctx.close()
