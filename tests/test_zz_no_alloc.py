"""The entry point that allocates nothing (selsync_grad_norm_sq_noalloc), called through the C ABI and
checked against the existing entry point it is a variant of (selsync_track_grad_change) and against
the CPU oracle: squared gradient norms within 1e-5 relative (the bar for norms), on two calls in a
row, the second with a smaller input, so stale contents of the shared device array would show."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from oracle import selsync_oracle as O                          # noqa: E402
from paper_2307_07950_amd import workloads as W                 # noqa: E402
from tests import parity_util as PU                             # noqa: E402

NORM_RTOL = 1e-5


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2307_07950_amd import binding
    return binding


def _case(B, numel, K, mixed, seed, gs, misalign=0):
    """Norms of one seeded input from the allocation-free entry point, the existing one and the oracle."""
    r = np.random.default_rng(seed)
    grads = []
    for k in range(K):
        gk = [(r.standard_normal(n) * 10.0 ** r.uniform(-3, 0)).astype(np.float32) for n in numel]
        grads.append([W.round_to_bf16_bits(a) for a in gk] if mixed else gk)
    ls = PU.LockStep(B, numel, K, delta=0.3, mixed=mixed, misalign=misalign, seed=seed)
    ls.bind_grads(0, grads)
    out = torch.full((K,), -1.0, dtype=torch.float64, device="cuda")
    # raw C-ABI call: host descriptors, device pointers, no context and no plan
    arr, keep = B._marshal_lists(ls.d_grads[0])
    stream = torch.cuda.current_stream().cuda_stream
    rc = B.selsync_grad_norm_sq_noalloc(arr, K, gs, ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(stream))
    assert rc == B.SELSYNC_OK
    got = out.cpu().tolist()
    ref = ls.ctx.track_grad_change(ls.plans[0], gs, blocking=True).norm_sq
    want = [O.norm_sq(grads[k], gs) for k in range(K)]
    ls.close()
    return got, ref, want


def _check(got, ref, want):
    for k in range(len(want)):
        assert got[k] == pytest.approx(ref[k], rel=NORM_RTOL)      # against the existing entry point: the bar
        assert got[k] == pytest.approx(want[k], rel=NORM_RTOL)     # against the oracle: the bar
        assert got[k] == pytest.approx(want[k], rel=1e-12)         # fp64 accumulation: far inside it


@pytest.mark.parametrize("mixed", [False, True])
def test_two_calls_in_a_row_the_second_smaller(B, mixed):
    # first call: several launches' worth of tensors (more than 64), ragged tails, empty tensors, pieces
    # beyond one tile; second call: a much smaller input that reuses the low slots of the device array
    big = [70001, 5, 0, 4096, 4097, 300000] + [1000 + 37 * i for i in range(70)]
    small = [5000, 3, 0, 8193]
    first = _case(B, big, 4, mixed, seed=900, gs=0.37)
    second = _case(B, small, 2, mixed, seed=901, gs=1.0)
    _check(*first)
    _check(*second)
    # and again the big one: same bits as the first time (fixed slots, fixed order)
    again = _case(B, big, 4, mixed, seed=900, gs=0.37)
    assert [x.hex() for x in again[0]] == [x.hex() for x in first[0]]


def test_unaligned_tensors_zero_and_constant_gradients(B):
    got, ref, want = _case(B, [70001, 33, 4099], 3, False, seed=902, gs=1.0, misalign=1)
    _check(got, ref, want)
    got, ref, want = _case(B, [70001, 33, 4099], 3, True, seed=903, gs=2.0, misalign=3)
    _check(got, ref, want)
    n = [100000, 33]
    z = [torch.zeros(m, device="cuda") for m in n]
    c = [torch.full((m,), 0.5, device="cuda") for m in n]
    out = torch.empty(2, dtype=torch.float64, device="cuda")
    B.grad_norm_sq_noalloc([z, c], out, 1.0)
    assert out.cpu().tolist() == [0.0, sum(n) * 0.25]
    # a worker list of only empty tensors, and no tensors at all
    out1 = torch.full((1,), 7.0, dtype=torch.float64, device="cuda")
    B.grad_norm_sq_noalloc([[torch.zeros(0, device="cuda")]], out1, 1.0)
    assert out1.item() == 0.0
    out1.fill_(7.0)
    B.grad_norm_sq_noalloc([[]], out1, 1.0)
    assert out1.item() == 0.0


def test_can_be_recorded_into_a_hip_graph_and_replayed(B):
    """Callers under graph capture are who the entry point is for: record it once, replay it several times with
    eager work and synchronisations in between, and compare every replay with an eager call on the same data."""
    K, numel = 3, [70001, 33, 4099, 0]
    gen = torch.Generator(device="cuda").manual_seed(904)
    grads = [[torch.randn(n, device="cuda", generator=gen) * 0.01 for n in numel] for _ in range(K)]
    out_g = torch.full((K,), -1.0, dtype=torch.float64, device="cuda")
    out_e = torch.full((K,), -1.0, dtype=torch.float64, device="cuda")
    B.grad_norm_sq_noalloc(grads, out_e, 0.5)          # first call on this GPU outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.grad_norm_sq_noalloc(grads, out_g, 0.5)
    torch.cuda.synchronize()
    assert out_g.cpu().tolist() == [-1.0] * K          # the capture itself runs nothing
    for rep in range(4):
        for k in range(K):                             # eager work between replays: new gradient values in place
            for x in grads[k]:
                x.mul_(1.0 + 0.25 * (rep + k))
        g.replay()
        torch.cuda.synchronize()
        B.grad_norm_sq_noalloc(grads, out_e, 0.5)
        torch.cuda.synchronize()
        assert [x.hex() for x in out_g.cpu().tolist()] == [x.hex() for x in out_e.cpu().tolist()]
        want = [O.norm_sq([PU.to_host(x) for x in grads[k]], 0.5) for k in range(K)]
        for k in range(K):
            assert out_g[k].item() == pytest.approx(want[k], rel=1e-12)
    del g


def test_limits_and_argument_errors(B):
    out = torch.zeros(65, dtype=torch.float64, device="cuda")
    g = [torch.zeros(16, device="cuda")]

    def status(lists, K=None, o=out):
        arr, keep = B._marshal_lists(lists)
        return B.selsync_grad_norm_sq_noalloc(arr, len(lists) if K is None else K, 1.0,
                                              ctypes.c_void_p(o.data_ptr()), None)

    assert status([g] * 65) == B.SELSYNC_ERR_TOO_LARGE                     # more than 64 workers
    assert status([g] * 64) == B.SELSYNC_OK
    # more pieces than the device array has slots: 2^20 + 1 tensors of one element each would do, so
    # do it with descriptors that point at the same small tensor (read-only inputs may alias)
    many = [g[0][:1]] * ((1 << 20) + 1)
    assert status([many]) == B.SELSYNC_ERR_TOO_LARGE
    assert status([[g[0][:1]] * 1000]) == B.SELSYNC_OK
    assert status([g, [torch.zeros(17, device="cuda")]]) == B.SELSYNC_ERR_SHAPE_MISMATCH
    assert status([g, [torch.zeros(16, device="cuda", dtype=torch.bfloat16)]]) == B.SELSYNC_ERR_DTYPE
    assert status([g], K=0) == B.SELSYNC_ERR_INVALID_ARG
    assert B.selsync_grad_norm_sq_noalloc(None, 1, 1.0, ctypes.c_void_p(out.data_ptr()), None) == B.SELSYNC_ERR_INVALID_ARG
    arr, keep = B._marshal_lists([g])
    assert B.selsync_grad_norm_sq_noalloc(arr, 1, 1.0, None, None) == B.SELSYNC_ERR_INVALID_ARG
    host = torch.zeros(16)
    d = (B.selsync_tensor * 1)()
    d[0].data, d[0].numel, d[0].dtype = host.data_ptr(), 16, B.SELSYNC_F32
    lst = (B.selsync_tensor_list * 1)()
    lst[0].tensors, lst[0].count = d, 1
    assert B.selsync_grad_norm_sq_noalloc(lst, 1, 1.0, ctypes.c_void_p(out.data_ptr()), None) == B.SELSYNC_ERR_NOT_DEVICE_MEM
    # a descriptor that claims more elements than its allocation holds is refused on the host
    big = torch.zeros(1 << 22, device="cuda")          # its own 16 MiB allocation
    d[0].data, d[0].numel = big.data_ptr(), (1 << 22) + (1 << 26)
    rc = B.selsync_grad_norm_sq_noalloc(lst, 1, 1.0, ctypes.c_void_p(out.data_ptr()), None)
    assert rc in (B.SELSYNC_ERR_INVALID_ARG, B.SELSYNC_ERR_TOO_LARGE)
    torch.cuda.synchronize()
