"""Parity of the further entry points with the oracle (needs an MI355X): per-component sync
periods (Algorithm 1: t mod H_i == 0), per-component neighbour counts, the final model average
(Algorithm 1, RETURN) and the gossip-MA branch at benchmark size.  All calls go through the
C ABI."""
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


@pytest.mark.parametrize("sampling", [B.SAMPLING_SEPARATE, B.SAMPLING_IN_KERNEL])
@pytest.mark.parametrize("K,q,sizes,periods", [
    (8, 2, [3000, 1, 4099, 0, 70000, 513], [4, 1, 2, 3, 8, 1]),                 # mixed: several runs
    (16, 3, [700] * 40, [1 + (i % 3) for i in range(40)]),                        # scattered
    (4, 1, [5000, 5000, 5000], [2, 2, 2]),                                        # nothing active on odd steps
    (64, 4, [4096] * 6 + [50000], [128] * 6 + [16]),                              # the paper's (16,128): one run
    (16, [3, 1, 2, 6, 0], [5000, 300, 70001, 12, 9000], [2, 3, 1, 4, 6]),         # periods and q per component
])
def test_sync_step_honours_per_component_periods(K, q, sizes, periods, sampling):
    _need_gpu()
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    stride = (P + 63) // 64 * 64
    seed = 77
    pl = B.Plan(off, K, q, 0, seed=seed, periods=periods, sampling=sampling)
    assert pl.info.has_periods == 1
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
    # a plan without periods: sync_step is the plain sync of round = step
    plain = B.Plan(off, K, q, 0, seed=seed, sampling=sampling)
    a = [t.clone() for t in dev]
    plain.sync_step(*dev, stride, 0.9, 1.0, B.MODE_PAPER, 5, None)
    plain.sync(*a, stride, 0.9, 1.0, B.MODE_PAPER, 5, None)
    torch.cuda.synchronize()
    for x, y in zip(dev, a):
        assert torch.equal(x, y)
    pl.destroy()
    plain.destroy()


def test_sync_step_when_components_that_are_not_due_lie_between_due_ones():
    # the sampler launch spans the first to the last due component and skips the ones in between
    _need_gpu()
    K, q = 8, 2
    sizes = [4000] * 6
    periods = [1, 4, 1, 1, 4, 1]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    stride = int(off[-1])
    pl = B.Plan(off, K, q, 0, seed=5, periods=periods, sampling=B.SAMPLING_SEPARATE)
    dev = list(_state(K, stride, 1))
    host = [t.cpu().numpy().copy() for t in dev]
    for t in (4, 5, 6, 8):
        pl.sync_step(*dev, stride, 0.9, 1.0, 1, t, None)
        oracle.sync(off, K, pl.info.p, q, 5, t, *host, np.float32(0.9), np.float32(1.0), 1,
                    active=(t % np.asarray(periods) == 0).astype(np.uint8))
    torch.cuda.synchronize()
    for d, h in zip(dev, host):
        assert (d.cpu().numpy() == h).all()
    pl.destroy()


@pytest.mark.parametrize("layout", ["blocked", "separate"])
def test_paper_shaped_workload_with_the_16_128_schedule_and_per_component_q(layout):
    # Section 3.2's 16-component split, Section 3.3's 16-GPU setting (p, q) = (3, 2) and periods
    # (16, 128); the second plan lets the embedding shards ask 3 neighbours and the tails 1
    _need_gpu()
    w = W.get("paper_shaped")
    off = W.component_offsets(w)
    m = len(off) - 1
    H = W.periods(w)
    assert m == 16 and H.tolist() == [128] * 8 + [16] * 8
    for q in (w.q, [3] * 8 + [2] * 3 + [1] * 5):
        pl = B.Plan(off, w.K, q, w.p, seed=w.seed, periods=H)
        assert pl.info.p == 3 and pl.info.q == (2 if np.ndim(q) == 0 else 3)
        st = W.init_state(w, DEV, layout=layout, plan=pl)
        T = pl.info.tile_columns_blocked if layout == "blocked" else pl.info.tile_columns
        cols, red = W.tile_columns(off, 4 * T * 64, seed=1)             # one element per 64 tiles
        idx = torch.from_numpy(cols).to(DEV)
        host = [st.gather(a, idx).cpu().numpy().copy() for a in range(3)]
        for t in (16, 32, 112, 128, 144, 256):
            if layout == "separate":
                pl.sync_step(*st.arrays, st.worker_stride, w.eta, w.zeta, w.mode, t, torch.cuda.current_stream())
            else:
                pl.sync_step_state(st.desc(), w.eta, w.zeta, w.mode, t, torch.cuda.current_stream())
            oracle.sync(red, w.K, 3, q, w.seed, t, *host, np.float32(w.eta), np.float32(w.zeta), w.mode,
                        active=(t % H == 0).astype(np.uint8))
        torch.cuda.synchronize()
        for a, name in enumerate(("theta", "omega", "delta")):
            assert (st.gather(a, idx).cpu().numpy() == host[a]).all(), (name, q)
        pl.destroy()
        del st
        torch.cuda.empty_cache()


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
    # the same values in a blocked placement (smallest legal block, gaps, aligned and not)
    Bf = pl.info.min_block_floats
    e = torch.arange(P, device=DEV)
    for ws, gap, sh in ((Bf, 0, 0), (Bf + 4, 8, 0), (Bf, 0, 1)):
        bs = (K - 1) * ws + Bf + gap
        nb = -(-P // Bf)
        arena = torch.randn(sh + nb * bs + 8, generator=g, device=DEV)
        ix = (sh + (e // Bf) * bs + e % Bf)[None, :] + torch.arange(K, device=DEV)[:, None] * ws
        arena[ix.reshape(-1)] = theta[:, :P].reshape(-1)
        out.fill_(7.0)
        pl.final_average_state(B.make_state(arena[sh:], None, None, ws, Bf, bs), out, None)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got[:P] == want).all() and (got[P:] == 7.0).all(), (ws, gap, sh)
    pl.destroy()


@pytest.mark.parametrize("layout", ["blocked", "separate"])
def test_final_average_at_benchmark_size(layout):
    _need_gpu()
    w = W.get(2)
    off = W.component_offsets(w)
    P = int(off[-1])
    pl = B.Plan(off, w.K, w.q, w.p, seed=0)
    st = W.DeviceState(w.K, P, DEV, layout, plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    (st.arena if st.arena is not None else st.arrays[0]).normal_(0, 0.02, generator=g)
    out = torch.empty(P, device=DEV)
    if layout == "separate":
        pl.final_average(st.arrays[0], st.worker_stride, out, None)
    else:
        pl.final_average_state(st.desc(gossip_ma=True), out, None)
    torch.cuda.synchronize()
    cols, _ = W.tile_columns(off, 4 * 256, seed=3)                       # one element per 1024
    idx = torch.from_numpy(cols).to(DEV)
    sub = np.ascontiguousarray(st.gather(0, idx).cpu().numpy())
    assert (out.index_select(0, idx).cpu().numpy() == oracle.final_average(sub)).all()
    pl.destroy()


@pytest.mark.parametrize("layout", ["blocked", "rows"])
def test_gossip_ma_at_benchmark_size(layout):
    # Algorithm 1's gossip-MA branch on the large-vocabulary model: theta' = average; the slots are not passed
    _need_gpu()
    w = W.get(3)
    off = W.component_offsets(w)
    P = int(off[-1])
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    st = W.DeviceState(w.K, P, DEV, layout, plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    st.arena.normal_(0, 0.02, generator=g)
    others = [st.gather(a, torch.arange(0, P, 100003, device=DEV)).clone() for a in (1, 2)]
    T = pl.info.tile_columns_blocked if layout == "blocked" else pl.info.tile_columns
    cols, red = W.tile_columns(off, 4 * T, seed=5)                       # an element of every tile
    idx = torch.from_numpy(cols).to(DEV)
    host = st.gather(0, idx).cpu().numpy().copy()
    for r in range(3):
        pl.sync_state(st.desc(gossip_ma=True), 0.0, 1.0, B.MODE_GOSSIP_MA, r, None)
        oracle.sync(red, w.K, pl.info.p, w.q, w.seed, r, host, None, None, np.float32(0), np.float32(1), 3)
    torch.cuda.synchronize()
    assert (st.gather(0, idx).cpu().numpy() == host).all()
    for a, before in zip((1, 2), others):                               # omega and Delta were not touched
        assert torch.equal(st.gather(a, torch.arange(0, P, 100003, device=DEV)), before)
    pl.destroy()


def test_full_size_every_element_all_neighbours_is_the_global_mean():
    # q = K-1 (every other worker): Section 2.2's degenerate case without gossip.  Every worker's
    # average is then the same ascending-id sum over all workers times fl(1/K), which plain
    # elementwise torch ops reproduce operation for operation: checked on EVERY element of the
    # large-vocabulary model, in the benchmark's blocked placement.
    _need_gpu()
    w = W.get(2)
    off = W.component_offsets(w)
    P = int(off[-1])
    pl = B.Plan(off, w.K, w.K - 1, -1, seed=0)
    st = W.DeviceState(w.K, P, DEV, "blocked", plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(11)
    st.arena.normal_(0, 0.02, generator=g)
    theta = st.arrays[0]                                    # [K, blocks, B] view
    s = theta[0].clone()
    for k in range(1, w.K):
        s += theta[k]                                       # one rounded fp32 add per worker, ascending
    s *= torch.tensor(1.0, device=DEV) / torch.tensor(float(w.K), device=DEV)
    for r in (0, 1):                                        # forward and backward sweep
        pl.sync_state(st.desc(gossip_ma=True), 0.0, 1.0, B.MODE_GOSSIP_MA, r, None)
        torch.cuda.synchronize()
        flat = s.reshape(-1)[:P]
        for k in range(w.K):
            assert torch.equal(theta[k].reshape(-1)[:P], flat), f"worker {k} round {r}"
        if r == 0:                                          # all workers equal now: the next mean of K equal
            t2 = s.clone()                                  # values, again op for op
            for k in range(1, w.K):
                t2 += s
            s = t2 * (torch.tensor(1.0, device=DEV) / torch.tensor(float(w.K), device=DEV))
    pl.destroy()


def test_full_size_every_element_invariants_of_one_sync():
    # Properties that hold at any size, checked on every element of config 3 (2,127 components):
    # the neighbour average lies between the workers' min and max; omega' = omega + Delta';
    # theta' = omega' + eta*Delta' (the restart statement), the latter two bit for bit.
    _need_gpu()
    w = W.get(3)
    off = W.component_offsets(w)
    P = int(off[-1])
    st = W.init_state(w, DEV, layout="separate")
    theta, omega, delta = st.arrays
    stride = st.worker_stride
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


def test_sync_step_on_blocked_state_with_scattered_periods_and_per_component_q():
    # the one-launch path (workgroups of components that are not due return at once) and the
    # one-run path, on the blocked arena, with a different q per component
    _need_gpu()
    K = 16
    sizes = [9000, 300, 70001, 12, 40000, 8192, 1]
    q = [3, 1, 2, 6, 0, 4, 2]
    periods = [2, 3, 1, 4, 6, 2, 3]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    for sampling in (B.SAMPLING_SEPARATE, B.SAMPLING_IN_KERNEL):
        pl = B.Plan(off, K, q, 0, seed=31, periods=periods, sampling=sampling)
        st = W.DeviceState(K, P, DEV, "blocked", plan=pl)
        g = torch.Generator(device=DEV)
        g.manual_seed(8)
        st.arena.normal_(0, 0.05, generator=g)
        junk = st.padding(0).clone()
        host = [st.to_host(a) for a in range(3)]
        for t in (1, 2, 3, 4, 6, 8, 9, 12):
            pl.sync_step_state(st.desc(), 0.9, 1.0, B.MODE_PAPER, t, None)
            oracle.sync(off, K, pl.info.p, q, 31, t, *host, np.float32(0.9), np.float32(1.0), 1,
                        active=(t % np.asarray(periods) == 0).astype(np.uint8))
        torch.cuda.synchronize()
        for a, name in enumerate(("theta", "omega", "delta")):
            assert (st.to_host(a) == host[a]).all(), (name, sampling)
        assert torch.equal(st.padding(0), junk)
        pl.destroy()


def test_caller_table_with_per_component_q_ignores_entries_beyond_q_i():
    _need_gpu()
    K, q = 8, [1, 3, 0, 2]
    off = np.array([0, 700, 20000, 20001, 33000], dtype=np.int64)
    P = int(off[-1])
    pl = B.Plan(off, K, q, 2, seed=3)
    nbr = oracle.neighbour_table(4, K, 2, q, seed=3, round=7)
    junk = nbr.copy()
    for i, qi in enumerate(q):
        junk[i, :, qi:] = 12345 + i                            # not worker ids
    for layout in ("separate", "blocked"):
        st = W.DeviceState(K, P, DEV, layout, plan=pl)
        g = torch.Generator(device=DEV)
        g.manual_seed(2)
        for buf in ([st.arena] if st.arena is not None else st.arrays):
            buf.normal_(0, 0.05, generator=g)
        host = [st.to_host(a) for a in range(3)]
        table = torch.from_numpy(junk).to(DEV)
        if layout == "separate":
            pl.sync_table(table, *st.arrays, st.worker_stride, 0.9, 1.0, B.MODE_PAPER, None)
        else:
            pl.sync_table_state(table, st.desc(), 0.9, 1.0, B.MODE_PAPER, None)
        oracle.sync_table(off, nbr, *host, np.float32(0.9), np.float32(1.0), 1, q=q)
        torch.cuda.synchronize()
        for a in range(3):
            assert (st.to_host(a) == host[a]).all(), (layout, a)
    pl.destroy()


def test_final_average_on_the_rows_arena():
    _need_gpu()
    K, P = 16, 300001
    pl = B.Plan([0, 1000, P], K, 2)
    st = W.DeviceState(K, P, DEV, "rows", plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    st.arena.normal_(0, 0.05, generator=g)
    out = torch.full((P + 3,), -1.0, device=DEV)
    pl.final_average_state(st.desc(gossip_ma=True), out, None)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got[:P] == oracle.final_average(st.to_host(0))).all() and (got[P:] == -1.0).all()
    pl.destroy()
