"""Parity of the further entry points with the oracle (needs an MI355X): per-component sync
periods (Algorithm 1: t mod H_i == 0), the final model average (Algorithm 1, RETURN) and the
gossip-MA branch at benchmark size.  All calls go through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_1909_09010_amd import binding as B
from paper_1909_09010_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _state(K, stride, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    w0 = torch.randn(stride, generator=g, device=DEV) * 0.05
    theta = (w0 + torch.randn((K, stride), generator=g, device=DEV) * 0.01).contiguous()
    omega = w0.repeat(K, 1).contiguous()
    delta = (torch.randn((K, stride), generator=g, device=DEV) * 0.001).contiguous()
    return theta, omega, delta


@pytest.mark.parametrize("K,q,sizes,periods", [
    (8, 2, [3000, 1, 4099, 0, 70000, 513], [4, 1, 2, 3, 8, 1]),                 # mixed, few runs
    (16, 3, [700] * 40, [1 + (i % 3) for i in range(40)]),                        # scattered: device-side check
    (4, 1, [5000, 5000, 5000], [2, 2, 2]),                                        # nothing active on odd steps
    (64, 4, [4096] * 6 + [50000], [128] * 6 + [16]),
])
def test_sync_step_honours_per_component_periods(K, q, sizes, periods):
    _need_gpu()
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    stride = (P + 63) // 64 * 64
    seed = 77
    pl = B.Plan(off, K, q, 0, seed=seed)
    pl.set_periods(periods)
    dev = list(_state(K, stride, 3))
    host = [t.cpu().numpy().copy() for t in dev]
    H = np.asarray(periods)
    steps = [1, 2, 3, 4, 6, 8, 12, 16, 24, 128, 129]
    for t in steps:
        pl.sync_step(*dev, stride, 0.9, 1.0, B.MODE_PAPER, t, torch.cuda.current_stream())
        active = (t % H == 0).astype(np.uint8)
        oracle.sync(off, K, pl.info.p, q, seed, t, *host, np.float32(0.9), np.float32(1.0), 1, active=active)
        dev[0] += 0.001                                          # local steps in between
        host[0] += np.float32(0.001)
    torch.cuda.synchronize()
    for name, d, h in zip(("theta", "omega", "delta"), dev, host):
        got = d.cpu().numpy()
        np.testing.assert_allclose(got, h, rtol=1e-6, atol=1e-7, err_msg=name)
        assert (got == h).all(), name
    # clearing the periods gives back the plain sync
    pl.set_periods(None)
    a = [t.clone() for t in dev]
    pl.sync_step(*dev, stride, 0.9, 1.0, B.MODE_PAPER, 5, None)
    pl.sync(*a, stride, 0.9, 1.0, B.MODE_PAPER, 5, None)
    torch.cuda.synchronize()
    for x, y in zip(dev, a):
        assert torch.equal(x, y)
    with pytest.raises(B.GbmufError):
        pl.set_periods([0] * len(periods))
    pl.destroy()


def test_paper_shaped_workload_with_the_16_128_schedule():
    _need_gpu()
    w = W.get("paper_shaped")
    off = W.component_offsets(w)
    P = int(off[-1])
    m = len(off) - 1
    H = W.periods(w)
    assert m == 16 and H.tolist() == [128] * 8 + [16] * 8
    theta, omega, delta = W.init_state(w, DEV)
    stride = theta.stride(0)
    cols, red = W.sample_columns(off, seed=1)
    idx = torch.from_numpy(cols).to(DEV)
    host = [t.index_select(1, idx).cpu().numpy().copy() for t in (theta, omega, delta)]
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    assert pl.info.p == 3 and pl.info.q == 2
    pl.set_periods(H)
    for t in (16, 32, 112, 128, 144, 256):
        pl.sync_step(theta, omega, delta, stride, w.eta, w.zeta, w.mode, t, torch.cuda.current_stream())
        oracle.sync(red, w.K, 3, w.q, w.seed, t, *host, np.float32(w.eta), np.float32(w.zeta), w.mode,
                    active=(t % H == 0).astype(np.uint8))
    torch.cuda.synchronize()
    for name, d, h in zip(("theta", "omega", "delta"), (theta, omega, delta), host):
        got = d.index_select(1, idx).cpu().numpy()
        assert (got == h).all(), name
    pl.destroy()


@pytest.mark.parametrize("K,P,pad,shift", [(8, 100003, 1, 0), (16, 65536, 0, 0), (5, 777, 3, 0), (64, 4096, 0, 0),
                                            (1, 50, 2, 0), (8, 100003, 5, 1), (3, 3, 1, 0)])
def test_final_average_matches_oracle(K, P, pad, shift):
    _need_gpu()
    stride = (P + 3) // 4 * 4 + pad
    g = torch.Generator(device=DEV)
    g.manual_seed(K + P)
    buf = torch.randn(K * stride + 8, generator=g, device=DEV)
    theta = buf[shift:shift + K * stride].view(K, stride)
    out = torch.full((P + 4,), 7.0, device=DEV)
    pl = B.Plan([0, P], K, 0, 0, seed=0)
    pl.final_average(theta, stride, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    want = oracle.final_average(np.ascontiguousarray(theta.cpu().numpy()), P)
    got = out.cpu().numpy()
    assert (got[:P] == want).all()
    assert (got[P:] == 7.0).all()
    with pytest.raises(B.GbmufError):
        pl.final_average(theta, P - 1, out)
    pl.destroy()


def test_final_average_at_benchmark_size():
    _need_gpu()
    w = W.get(2)
    off = W.component_offsets(w)
    P = int(off[-1])
    theta, _, _, stride = W.alloc_state(w.K, P, DEV)
    theta.normal_(0, 0.02)
    out = torch.empty(P, device=DEV)
    pl = B.Plan(off, w.K, w.q, w.p, seed=0)
    pl.final_average(theta, stride, out, None)
    torch.cuda.synchronize()
    cols, _ = W.sample_columns(off, seed=3)
    idx = torch.from_numpy(cols).to(DEV)
    sub = np.ascontiguousarray(theta.index_select(1, idx).cpu().numpy())
    assert (out.index_select(0, idx).cpu().numpy() == oracle.final_average(sub)).all()
    pl.destroy()


def test_gossip_ma_at_benchmark_size():
    # Algorithm 1's gossip-MA branch on the large-vocabulary model: theta' = average; the slots are not passed
    _need_gpu()
    w = W.get(3)
    off = W.component_offsets(w)
    P = int(off[-1])
    theta, _, _, stride = W.alloc_state(w.K, P, DEV)
    theta.normal_(0, 0.02)
    cols, red = W.sample_columns(off, seed=5)
    idx = torch.from_numpy(cols).to(DEV)
    host = theta.index_select(1, idx).cpu().numpy().copy()
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    for r in range(3):
        pl.sync(theta, None, None, stride, 0.0, 1.0, B.MODE_GOSSIP_MA, r, None)
        oracle.sync(red, w.K, pl.info.p, w.q, w.seed, r, host, None, None, np.float32(0), np.float32(1), 3)
    torch.cuda.synchronize()
    assert (theta.index_select(1, idx).cpu().numpy() == host).all()
    pl.destroy()


def test_full_size_every_element_all_neighbours_is_the_global_mean():
    # q = K-1 (every other worker): Section 2.2's degenerate case without gossip.  Every worker's
    # average is then the same ascending-id sum over all workers times fl(1/K), which plain
    # elementwise torch ops reproduce operation for operation: checked on EVERY element of the
    # large-vocabulary model, in the benchmark's HBM-spanning layout.
    _need_gpu()
    w = W.get(2)
    off = W.component_offsets(w)
    P = int(off[-1])
    span = W.default_span_bytes(DEV, 3 * w.K * W.padded_stride(P) * 4)
    theta, _, _, stride = W.alloc_state(w.K, P, DEV, span_bytes=span)
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    for k in range(w.K):
        theta[k].normal_(0, 0.02, generator=g)
    s = theta[0].clone()
    for k in range(1, w.K):
        s += theta[k]                                       # one rounded fp32 add per worker, ascending
    s *= torch.tensor(1.0, device=DEV) / torch.tensor(float(w.K), device=DEV)
    pl = B.Plan(off, w.K, w.K - 1, -1, seed=0)
    pl.sync(theta, None, None, stride, 0.0, 1.0, B.MODE_GOSSIP_MA, 0, None)
    torch.cuda.synchronize()
    for k in range(w.K):
        assert torch.equal(theta[k, :P], s[:P]), f"worker {k}"
    pl.destroy()


def test_full_size_every_element_invariants_of_one_sync():
    # Properties that hold at any size, checked on every element of config 3 (2,127 components):
    # the neighbour average lies between the workers' min and max; omega' = omega + Delta';
    # theta' = omega' + eta*Delta' (the restart statement), the latter two bit for bit.
    _need_gpu()
    w = W.get(3)
    off = W.component_offsets(w)
    P = int(off[-1])
    theta, omega, delta = W.init_state(w, DEV)
    stride = theta.stride(0)
    lo, hi = theta.min(dim=0).values, theta.max(dim=0).values
    omega_before = omega.clone()
    avg = theta.clone()
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    pl.sync(avg, None, None, stride, 0.0, 1.0, B.MODE_GOSSIP_MA, 0, None)
    slack = 4 * torch.finfo(torch.float32).eps * torch.maximum(lo.abs(), hi.abs())
    assert bool(((avg >= lo - slack) & (avg <= hi + slack))[:, :P].all())
    assert float((avg - theta)[:, :P].abs().max()) > 1e-3                   # and it did average
    del lo, hi, slack
    eta = 0.9
    pl.sync(theta, omega, delta, stride, eta, w.zeta, B.MODE_PAPER, 0, None)
    torch.cuda.synchronize()
    assert torch.equal(omega[:, :P], (omega_before + delta)[:, :P])
    step = delta * torch.tensor(eta, dtype=torch.float32, device=DEV)       # rounded product, then rounded add
    assert torch.equal(theta[:, :P], (omega + step)[:, :P])
    # zeta = 1: omega' equals the average up to the rounding of three additions
    assert float((omega - avg)[:, :P].abs().max()) < 1e-6
    pl.destroy()
