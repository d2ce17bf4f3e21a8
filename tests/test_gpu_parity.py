"""Parity of the HIP path with the CPU oracle (needs an MI355X; run with -m gpu).

Neighbour tables are compared bit for bit.  Parameters are compared element by element
with the fp32 writing of the oracle at the benchmark's tolerance (1e-6 relative, 1e-7
absolute); both sides perform the same IEEE operations in the same order, so the expected
difference is zero and the tests also require bit equality.  Every call goes through the C
ABI (ctypes binding).  State placements covered: three separate [K, stride] tensors, the
rows arena and the blocked arena (the benchmark's), plus hand-made blocked geometries.
"""
import dataclasses
import itertools

import numpy as np
import pytest

import oracle
from paper_1909_09010_amd import binding as B
from paper_1909_09010_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-6, 1e-7
DEV = "cuda:0"


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _to_host(*ts):
    return [t.detach().cpu().numpy().copy() for t in ts]


def _compare(dev_states, host_states, P, what=""):
    torch.cuda.synchronize()
    exact = 0
    total = 0
    for name, d, h in zip(("theta", "omega", "delta"), dev_states, host_states):
        if d is None:
            continue
        got = d.detach().cpu().numpy()
        np.testing.assert_allclose(got[:, :P], h[:, :P], rtol=RTOL, atol=ATOL, err_msg=f"{what} {name}")
        assert (got[:, P:] == h[:, P:]).all(), f"{what} {name}: padding was touched"
        exact += int((got[:, :P] == h[:, :P]).sum())
        total += got[:, :P].size
    return exact, total


def _random_state(K, P, stride, seed, delta_std=0.01):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    pad = torch.randn((K, stride), generator=g, device=DEV)          # padding holds junk on purpose
    w0 = torch.randn(stride, generator=g, device=DEV) * 0.05
    theta = w0 + torch.randn((K, stride), generator=g, device=DEV) * 0.01
    omega = w0.repeat(K, 1)
    delta = torch.randn((K, stride), generator=g, device=DEV) * delta_std
    for t in (theta, omega, delta):
        t[:, P:] = pad[:, P:]
    return theta.contiguous(), omega.contiguous(), delta.contiguous()


class BlockedArena:
    """A hand-made blocked placement of three [K, P] arrays inside one junk-filled arena:
    element (a, w, e) at base[a] + (e // Bf) * bs + w * ws + e % Bf (+ shift floats)."""

    def __init__(self, K, P, Bf, ws=None, bs=None, gap=0, shift=0, seed=0):
        self.K, self.P, self.Bf = K, P, Bf
        self.ws = Bf if ws is None else ws
        span = (K - 1) * self.ws + Bf
        self.bs = 3 * span + gap if bs is None else bs
        nb = max(1, -(-P // Bf))
        self.base = [shift, shift + span, shift + 2 * span]
        n = shift + (nb - 1) * self.bs + 3 * span + 8
        g = torch.Generator(device=DEV)
        g.manual_seed(seed)
        self.arena = torch.randn(n, generator=g, device=DEV)
        e = torch.arange(P, device=DEV)
        w = torch.arange(K, device=DEV)[:, None]
        self.idx = [(b + (e // Bf) * self.bs + e % Bf)[None, :] + w * self.ws for b in self.base]
        mask = torch.ones(n, dtype=torch.bool, device=DEV)
        for ix in self.idx:
            mask[ix.reshape(-1)] = False
        self.junk_mask = mask
        self.junk = self.arena[mask].clone()

    def put(self, arrays):
        for ix, a in zip(self.idx, arrays):
            self.arena[ix.reshape(-1)] = a[:, : self.P].reshape(-1)

    def get(self):
        return [self.arena[ix.reshape(-1)].view(self.K, self.P) for ix in self.idx]

    def desc(self, gossip_ma=False):
        p = [self.arena[b:] for b in self.base]
        return B.make_state(p[0], None if gossip_ma else p[1], None if gossip_ma else p[2], self.ws, self.Bf, self.bs)

    def junk_untouched(self):
        return torch.equal(self.arena[self.junk_mask], self.junk)


# --------------------------------------------------------------------------------------
# sampler
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("K,p,q,m", [(4, 1, 1, 9), (8, 2, 2, 9), (16, 3, 3, 2127), (64, 5, 4, 135), (64, -1, 63, 3),
                                     (5, 2, 3, 7), (12, 0, 2, 11), (2, 0, 1, 4), (16, 3, 6, 5), (33, 7, 9, 5),
                                     (128, -1, 20, 2), (1024, 0, 5, 2), (256, -1, 255, 1)])
def test_device_sampler_is_bit_exact(K, p, q, m):
    _need_gpu()
    off = np.arange(m + 1, dtype=np.int64) * 5
    for seed in (0, 0xDEADBEEFCAFEF00D):
        try:
            pl = B.Plan(off, K, q, p, seed=seed)
        except B.GbmufError as e:                       # the fused kernel's LDS limit, not the sampler's
            assert e.code == B.GBMUF_EUNSUPPORTED and K * (q + 1) > 16384
            return
        out = torch.full((m, K, q), -1, dtype=torch.int32, device=DEV)
        for rnd in (0, 1, 49, 2**32 + 3, 2**64 - 1):
            pl.neighbours_device(rnd, out, torch.cuda.current_stream())
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert (got == pl.neighbours_host(rnd)).all()
            assert (got == oracle.neighbour_table(m, K, pl.info.p, q, seed, rnd)).all()
        pl.destroy()


@pytest.mark.parametrize("K,p,q", [(8, 2, [0, 1, 2, 3, 4]), (16, 3, [6, 2, 2, 0, 1, 5] * 50), (4, 1, [1, 2, 0]),
                                   (64, -1, [63, 1, 7]), (16, 3, [2] * 8 + [3] * 8)])
def test_device_sampler_with_per_component_q_is_bit_exact(K, p, q):
    # device = host = oracle: three separately written samplers; rows end in -1 beyond q_i
    _need_gpu()
    m = len(q)
    off = np.arange(m + 1, dtype=np.int64) * 9
    pl = B.Plan(off, K, q, p, seed=77)
    out = torch.full((m, K, max(q)), 99, dtype=torch.int32, device=DEV)
    for rnd in (0, 5, 2**40 + 1):
        pl.neighbours_device(rnd, out, None)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got == pl.neighbours_host(rnd)).all()
        assert (got == oracle.neighbour_table(m, K, pl.info.p, q, 77, rnd)).all()
    pl.destroy()


# --------------------------------------------------------------------------------------
# arithmetic with enumerated tables
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_every_neighbour_assignment_on_K4(mode, blocked):
    _need_gpu()
    K, p, q = 4, 1, 1
    off = np.array([0, 5, 12], dtype=np.int64)
    P, stride = 12, 16
    pl = B.Plan(off, K, q, p, seed=0)
    theta0, omega0, delta0 = _random_state(K, P, stride, seed=mode)
    host0 = _to_host(theta0, omega0, delta0)
    arena = BlockedArena(K, P, pl.info.min_block_floats, seed=3) if blocked else None
    per_worker = [list(itertools.combinations(sorted(oracle.ring_candidates(w, K, p).tolist()), q)) for w in range(K)]
    slots = [per_worker[w] for _ in range(2) for w in range(K)]
    n = 0
    for combo in itertools.product(*slots):
        nbr = np.array(combo, dtype=np.int32).reshape(2, K, q)
        host = [h.copy() for h in host0]
        oracle.sync_table(off, nbr, *host, np.float32(0.9), np.float32(0.75), mode)
        if blocked:
            arena.put((theta0, omega0, delta0))
            pl.sync_table_state(torch.from_numpy(nbr).to(DEV), arena.desc(mode == 3), 0.9, 0.75, mode, None)
            dev = arena.get()
            host = [h[:, :P] for h in host]
        else:
            dev = [t.clone() for t in (theta0, omega0, delta0)]
            pl.sync_table(torch.from_numpy(nbr).to(DEV), *dev, stride, 0.9, 0.75, mode, torch.cuda.current_stream())
        exact, total = _compare(dev, host, P, f"table {n}")
        assert exact == total
        n += 1
    assert n == 256
    assert arena is None or arena.junk_untouched()


def test_unsorted_caller_table_gives_the_same_result():
    _need_gpu()
    K, q, m, P = 8, 3, 2, 100
    off = np.array([0, 33, 100], dtype=np.int64)
    pl = B.Plan(off, K, q, -1, seed=0)
    nbr = oracle.neighbour_table(m, K, K // 2, q, 3, 0)
    shuffled = nbr[:, :, ::-1].copy()
    a = _random_state(K, P, 128, 1)
    b = [t.clone() for t in a]
    pl.sync_table(torch.from_numpy(nbr).to(DEV), *a, 128, 0.9, 1.0, 1, None)
    pl.sync_table(torch.from_numpy(shuffled).to(DEV), *b, 128, 0.9, 1.0, 1, None)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


# --------------------------------------------------------------------------------------
# whole sync, small and ragged shapes, every code path
# --------------------------------------------------------------------------------------
SHAPES = [
    # K, p, q, offsets, stride_pad, base_shift (floats), rounds
    (4, 1, 1, [0, 5, 12, 12, 4099, 4100, 9001], 0, 0, 4),          # ragged, empty component, unaligned edges
    (4, 1, 1, [0, 5, 12, 12, 4099, 4100, 9001], 3, 0, 3),          # stride % 4 != 0: 4-byte path
    (4, 1, 1, [0, 5, 12, 12, 4099, 4100, 9001], 7, 1, 3),          # misaligned base: 4-byte path
    (8, 2, 2, [0, 70000, 70001, 140003], 1, 0, 3),                 # several tiles + ragged tail
    (16, 3, 3, [0, 2048, 133120, 135168, 150000], 0, 0, 3),
    (16, 3, 0, [0, 999, 5000], 0, 0, 3),                           # q = 0: purely local block momentum
    (16, 3, 6, [0, 999, 5000], 0, 0, 3),                           # q = 2p: local-BMUF, run-time q kernel
    (64, 5, 4, [0, 4096, 20000, 70001], 3, 0, 2),
    (64, -1, 63, [0, 300, 3001], 0, 0, 2),                         # every other worker: BMUF
    (5, 2, 3, [0, 17, 10000], 0, 0, 3),                            # K not a power of two
    (12, 0, 2, [0, 8000, 8001, 30000], 0, 0, 3),
    (1, 0, 0, [0, 100, 5000], 0, 0, 3),                            # a single worker
    (2, 0, 1, [0, 3, 50000], 0, 0, 3),
    (100, 0, 7, [0, 1000, 7001], 0, 0, 2),                         # tile narrower than a wavefront
    (1024, 0, 5, [0, 300, 1501], 0, 0, 2),                         # the largest K: 4 columns per tile
    (257, 0, 4, [0, 64, 2049], 0, 0, 2),
    (16, 3, [3, 0, 6, 1], [0, 2048, 33120, 35168, 50000], 0, 0, 3),   # a different q per component
    (8, 2, [4, 1, 2], [0, 70000, 70001, 140003], 1, 0, 3),
    (64, 5, [4, 10, 0], [0, 4096, 20000, 70001], 0, 0, 2),
]


@pytest.mark.parametrize("mode", [1, 0, 2, 3])
@pytest.mark.parametrize("K,p,q,off,pad,shift,rounds", SHAPES)
def test_sync_matches_oracle(K, p, q, off, pad, shift, rounds, mode):
    _need_gpu()
    off = np.asarray(off, dtype=np.int64)
    P = int(off[-1])
    stride = (P + 3) // 4 * 4 + pad
    seed = 1234 + K
    pl = B.Plan(off, K, q, p, seed=seed)
    big = _random_state(K, P + 0, stride + 0, seed=K * 7 + mode)
    if shift:
        # same rows, but every base pointer moved by `shift` floats inside a larger buffer
        dev = []
        for t in big:
            buf = torch.zeros(K * stride + 8, device=DEV)
            view = buf[shift:shift + K * stride].view(K, stride)
            view.copy_(t)
            dev.append(view)
    else:
        dev = list(big)
    host = _to_host(*dev)
    eta, zeta = 0.9, (1.0 if mode != 2 else 0.5)
    for r in range(rounds):
        args = dev if mode != 3 else [dev[0], None, None]
        pl.sync(*args, stride, eta, zeta, mode, r, torch.cuda.current_stream())
        hargs = host if mode != 3 else [host[0], None, None]
        oracle.sync(off, K, pl.info.p, q, seed, r, *hargs, np.float32(eta), np.float32(zeta), mode)
    exact, total = _compare(dev, host, P, f"K={K} q={q} mode={mode}")
    assert exact == total, f"{total - exact} of {total} elements differ in the last bits"
    pl.destroy()


# geometry of the blocked placement: (block as a multiple of the smallest legal one, worker stride
# beyond the block, gap between block groups, base shift in floats)
GEOMETRIES = [(1, 0, 0, 0), (4, 0, 0, 0), (2, 64, 128, 0), (1, 0, 0, 1), (2, 4, 12, 3), (1, 6, 2, 0)]


@pytest.mark.parametrize("geo", GEOMETRIES)
@pytest.mark.parametrize("K,p,q,off,pad,shift,rounds", [SHAPES[i] for i in (0, 3, 4, 6, 7, 9, 11, 14, 16, 18)])
def test_sync_matches_oracle_on_blocked_state(K, p, q, off, pad, shift, rounds, geo):
    _need_gpu()
    off = np.asarray(off, dtype=np.int64)
    P = int(off[-1])
    seed = 99 + K
    pl = B.Plan(off, K, q, p, seed=seed)
    mult, extra_ws, gap, base_shift = geo
    Bf = pl.info.min_block_floats * mult
    arena = BlockedArena(K, P, Bf, ws=Bf + extra_ws, gap=gap, shift=base_shift, seed=K)
    init = _random_state(K, P, P, seed=K + 11)
    for mode in (1, 3):
        arena.put(init)
        host = _to_host(*init)
        for r in range(rounds):
            pl.sync_state(arena.desc(mode == 3), 0.9, 1.0, mode, r, None)
            hargs = host if mode != 3 else [host[0], None, None]
            oracle.sync(off, K, pl.info.p, q, seed, r, *hargs, np.float32(0.9), np.float32(1.0), mode)
        torch.cuda.synchronize()
        got = arena.get()
        for name, g, h in zip(("theta", "omega", "delta"), got, host):
            assert (g.cpu().numpy() == h).all(), f"{name} mode {mode} geometry {geo}"
        assert arena.junk_untouched(), "floats outside the state were written"
    pl.destroy()


def test_state_copy_moves_between_placements():
    _need_gpu()
    K, P = 8, 70001
    pl = B.Plan([0, 30000, P], K, 2)
    src = _random_state(K, P, P + 3, seed=1)
    Bf = pl.info.min_block_floats
    for geo_args in (dict(), dict(ws=Bf + 8, gap=16), dict(shift=1)):
        arena = BlockedArena(K, P, Bf, seed=2, **geo_args)
        rows = B.make_state(*src, P + 3)
        pl.state_copy(arena.desc(), rows, 7, None)
        torch.cuda.synchronize()
        for g, s in zip(arena.get(), src):
            assert torch.equal(g, s[:, :P])
        assert arena.junk_untouched()
        back = [torch.full_like(s, 7.0) for s in src]
        pl.state_copy(B.make_state(*back, P + 3), arena.desc(), 5, None)       # theta and delta only
        torch.cuda.synchronize()
        assert torch.equal(back[0][:, :P], src[0][:, :P]) and torch.equal(back[2][:, :P], src[2][:, :P])
        assert bool((back[1] == 7.0).all()) and bool((back[0][:, P:] == 7.0).all())
    pl.destroy()


def test_tuning_options_do_not_change_a_bit():
    # tile shape, resident workgroups, sweep direction, cache hints and where the rows are drawn
    _need_gpu()
    K, q = 16, 3
    off = np.array([0, 50000, 50001, 300000], dtype=np.int64)
    P = 300000
    init = _random_state(K, P, P, seed=4)
    host = _to_host(*init)
    for r in range(3):
        oracle.sync(off, K, oracle.default_p(K), q, 5, r, *host, np.float32(0.9), np.float32(1.0), 1)
    options = [dict(), dict(tile=(256, 2), workgroups_per_cu=3), dict(tile=(1024, 1), workgroups_per_cu=1),
               dict(tile=(256, 8), sweep=B.SWEEP_FORWARD), dict(cache_hints=3, workgroups_per_cu=8),
               dict(sampling=B.SAMPLING_IN_KERNEL), dict(sampling=B.SAMPLING_SEPARATE, tile=(512, 4))]
    for opt in options:
        pl = B.Plan(off, K, q, 0, seed=5, **opt)
        rows = [t.clone() for t in init]
        arena = BlockedArena(K, P, pl.info.min_block_floats, seed=1)
        arena.put(init)
        for r in range(3):
            pl.sync(*rows, P, 0.9, 1.0, 1, r, None)
            pl.sync_state(arena.desc(), 0.9, 1.0, 1, r, None)
        torch.cuda.synchronize()
        for g, b, h in zip(rows, arena.get(), host):
            assert (g.cpu().numpy() == h).all() and (b.cpu().numpy() == h).all(), opt
        pl.destroy()


def test_denormals_signed_zeros_and_non_finite_values_propagate_like_the_oracle():
    # fp32 denormals are kept (no flush to zero), -0.0 keeps its sign where IEEE says so,
    # inf/nan propagate: compared bit for bit except for the payload of NaNs
    _need_gpu()
    K, q, off = 8, 2, np.array([0, 1000, 4100], dtype=np.int64)
    P, stride = 4100, 4160
    rng = np.random.default_rng(5)
    base = rng.normal(0, 2e-39, size=(3, K, stride)).astype(np.float32)         # denormal
    base[:, :, 10:20] = 0.0
    base[0, :, 20:30] = -0.0
    base[0, 3, 40] = np.inf
    base[0, 5, 41] = -np.inf
    base[1, 2, 42] = np.nan
    base[2, 1, 43] = np.float32(3e38)
    base[0, :, 50:60] = np.float32(3e38)                                          # the sum overflows
    assert (np.abs(base[0, :, 100:200]) < np.finfo(np.float32).tiny).mean() > 0.99
    pl = B.Plan(off, K, q, 0, seed=3)
    dev = [torch.from_numpy(b.copy()).to(DEV) for b in base]
    host = [b.copy() for b in base]
    for r in range(3):
        pl.sync(*dev, stride, 0.9, 1.0, 1, r, None)
        with np.errstate(all="ignore"):
            oracle.sync(off, K, pl.info.p, q, 3, r, *host, np.float32(0.9), np.float32(1.0), 1)
    torch.cuda.synchronize()
    for name, d, h in zip(("theta", "omega", "delta"), dev, host):
        got = d.cpu().numpy()
        nan = np.isnan(h)
        assert (np.isnan(got) == nan).all(), name
        assert (got.view(np.int32)[~nan] == h.view(np.int32)[~nan]).all(), name
    assert np.isnan(host[0]).any() and np.isinf(host[0]).any()
    assert ((np.abs(host[1]) < np.finfo(np.float32).tiny) & (host[1] != 0)).any()   # denormals survived
    pl.destroy()


def test_two_plans_on_two_streams_do_not_disturb_each_other():
    _need_gpu()
    K, q, off = 16, 3, np.array([0, 50000, 300000], dtype=np.int64)
    P = stride = 300000
    plans = [B.Plan(off, K, q, 0, seed=s) for s in (1, 2)]
    states = [list(_random_state(K, P, stride, 10 + i)) for i in range(2)]
    hosts = [_to_host(*st) for st in states]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for r in range(4):
        for pl, st, s in zip(plans, states, streams):
            pl.sync(*st, stride, 0.9, 1.0, 1, r, s)
    for s in streams:
        s.synchronize()
    for i, (pl, h) in enumerate(zip(plans, hosts)):
        for r in range(4):
            oracle.sync(off, K, pl.info.p, q, i + 1, r, *h, np.float32(0.9), np.float32(1.0), 1)
        exact, total = _compare(states[i], h, P, f"plan {i}")
        assert exact == total
        pl.destroy()


@pytest.mark.parametrize("K,q,P", [(16, 3, 150000), (16, 3, 3000001), (64, 4, 70001), (4, 1, 195048), (8, 2, 2500000),
                                   (16, [3, 1, 6], 150000)])
def test_in_kernel_sampling_and_the_sampler_kernel_give_identical_results(K, q, P):
    # small plans draw the neighbour rows inside the fused kernel, large ones launch the sampler
    # first; both ways (chosen through the plan description) must agree bitwise
    _need_gpu()
    off = np.array([0, P // 3, P // 3 + 1, P], dtype=np.int64)
    stride = (P + 63) // 64 * 64
    results = []
    for how in (B.SAMPLING_IN_KERNEL, B.SAMPLING_SEPARATE):
        pl = B.Plan(off, K, q, 0, seed=21, sampling=how)
        assert pl.info.in_kernel_sampling == (1 if how == B.SAMPLING_IN_KERNEL else 0)
        st = list(_random_state(K, P, stride, 9))
        for r in range(3):
            pl.sync(*st, stride, 0.9, 1.0, 1, r, None)
        torch.cuda.synchronize()
        results.append(st)
        pl.destroy()
    for x, y in zip(*results):
        assert torch.equal(x, y)
    host = _to_host(*_random_state(K, P, stride, 9))
    for r in range(3):
        oracle.sync(off, K, oracle.default_p(K), q, 21, r, *host, np.float32(0.9), np.float32(1.0), 1)
    exact, total = _compare(results[0], host, P, "in-kernel sampling")
    assert exact == total


def test_plans_with_different_lds_needs_coexist():
    # a plan with long neighbour rows (more LDS) made first must keep working after a plan with
    # short rows has been made for the same kernel
    _need_gpu()
    off = np.array([0, 3000, 9001], dtype=np.int64)
    K, P, stride = 64, 9001, 9216
    big = B.Plan(off, K, 40, -1, seed=1)             # run-time q kernel, 64*41 ids
    small = B.Plan(off, K, 8, -1, seed=1)            # same kernel (q+1 > 5), 64*9 ids
    for pl, q in ((big, 40), (small, 8), (big, 40)):
        st = list(_random_state(K, P, stride, 3))
        host = _to_host(*st)
        pl.sync(*st, stride, 0.9, 1.0, 1, 0, None)
        oracle.sync(off, K, K // 2, q, 1, 0, *host, np.float32(0.9), np.float32(1.0), 1)
        exact, total = _compare(st, host, P, f"q={q}")
        assert exact == total
    big.destroy()
    small.destroy()


def test_sync_equals_sync_table_with_the_sampled_table():
    _need_gpu()
    K, q, off = 16, 3, np.array([0, 1000, 66000], dtype=np.int64)
    pl = B.Plan(off, K, q, 0, seed=9)
    a = _random_state(K, 66000, 66048, 5)
    b = [t.clone() for t in a]
    nbr = torch.zeros((2, K, q), dtype=torch.int32, device=DEV)
    for r in range(3):
        pl.sync(*a, 66048, 0.9, 1.0, 1, r, None)
        pl.neighbours_device(r, nbr, None)
        pl.sync_table(nbr, *b, 66048, 0.9, 1.0, 1, None)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_rounds_are_stateless_resume_is_bit_identical_on_a_side_stream():
    _need_gpu()
    K, q, off = 8, 2, np.array([0, 5000, 20000], dtype=np.int64)
    pl = B.Plan(off, K, q, 0, seed=4)
    a = _random_state(K, 20000, 20000, 6)
    b = [t.clone() for t in a]
    for r in range(6):
        pl.sync(*a, 20000, 0.9, 1.0, 1, r, None)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        for r in range(3):
            pl.sync(*b, 20000, 0.9, 1.0, 1, r, s)
    s.synchronize()
    b = [t.cpu().to(DEV) for t in b]                                 # "checkpoint" round trip
    pl2 = B.Plan(off, K, q, 0, seed=4)
    for r in range(3, 6):
        pl2.sync(*b, 20000, 0.9, 1.0, 1, r, None)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_plain_c_program_on_the_c_abi_matches_the_oracle():
    # tests/abi_smoke.c: no Python, no torch; device memory from the HIP runtime
    _need_gpu()
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_smoke")
    if not os.path.exists(exe):
        pytest.skip("tests/abi_smoke has not been built (run __graft_entry__.build())")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.startswith("abi_smoke ok"), (r.stdout, r.stderr)


def test_sync_argument_errors():
    _need_gpu()
    pl = B.Plan([0, 64], K=4, q=1)
    t = torch.zeros((4, 64), device=DEV)
    for kw in (dict(worker_stride=63), dict(nesterov=4), dict(nesterov=-1)):
        args = dict(worker_stride=64, eta=0.9, zeta=1.0, nesterov=1, round=0)
        args.update(kw)
        with pytest.raises(B.GbmufError) as e:
            pl.sync(t, t.clone(), t.clone(), **args)
        assert e.value.code == B.GBMUF_EINVAL
    with pytest.raises(B.GbmufError):
        pl.sync(t, None, None, 64, 0.9, 1.0, 1, 0)
    with pytest.raises(B.GbmufError):
        pl.sync(None, t, t, 64, 0.9, 1.0, 1, 0)
    # overlapping arrays are refused, and nothing was written
    buf = torch.zeros(3 * 4 * 64, device=DEV)
    with pytest.raises(B.GbmufError) as e:
        pl.sync(buf, buf[32:], buf[2 * 256:], 64, 0.9, 1.0, 1, 0)
    assert e.value.code == B.GBMUF_EINVAL
    with pytest.raises(B.GbmufError) as e:
        pl.sync(buf, buf[256:], buf[256 + 63:], 64, 0.9, 1.0, 1, 0)
    assert e.value.code == B.GBMUF_EINVAL
    torch.cuda.synchronize()
    assert float(buf.abs().max()) == 0.0


# --------------------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------------------
def _sync(pl, st, w, r):
    if st.layout == "separate":
        t, o, d = st.arrays
        pl.sync(t, o, d, st.worker_stride, w.eta, w.zeta, w.mode, r, torch.cuda.current_stream())
    else:
        pl.sync_state(st.desc(), w.eta, w.zeta, w.mode, r, torch.cuda.current_stream())


def _run_full(w, layout, stride=None, drift_each_round=False):
    """Every element of the state, every round, against the oracle."""
    off = W.component_offsets(w)
    P = int(off[-1])
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    st = W.init_state(w, DEV, layout=layout, stride=stride, plan=pl)
    host = [st.to_host(a) for a in range(3)]
    pads = [st.padding(a).clone() for a in range(3)]
    m = len(off) - 1
    nbr = torch.zeros((m, w.K, w.q), dtype=torch.int32, device=DEV)
    for r in range(w.rounds):
        if drift_each_round and r > 0:
            for k in range(w.K):
                d = W.drift_row(w, DEV, P, r, k)
                st.add_to_row(0, k, d)
                host[0][k] += d.cpu().numpy()
        _sync(pl, st, w, r)
        pl.neighbours_device(r, nbr, torch.cuda.current_stream())
        oracle.sync(off, w.K, pl.info.p, w.q, w.seed, r, *host, np.float32(w.eta), np.float32(w.zeta), w.mode)
        torch.cuda.synchronize()
        assert (nbr.cpu().numpy() == oracle.neighbour_table(m, w.K, pl.info.p, w.q, w.seed, r)).all()
    for a, name in enumerate(("theta", "omega", "delta")):
        got = st.to_host(a)
        np.testing.assert_allclose(got, host[a], rtol=RTOL, atol=ATOL, err_msg=f"{w.name} {name}")
        assert (got == host[a]).all(), f"{w.name} {name}: elements differ in the last bits"
        assert torch.equal(st.padding(a), pads[a]), f"{w.name} {name}: padding was touched"
    pl.destroy()
    print(f"{w.name} [{layout}]: full state, {w.rounds} rounds, {3 * w.K * P} values compared after the last round, all bit-equal")


@pytest.mark.parametrize("layout", ["blocked", "rows", "separate"])
def test_config0_tiny_full_state_all_rounds(layout):
    _need_gpu()
    _run_full(W.get(0), layout, drift_each_round=True)


@pytest.mark.parametrize("layout", ["blocked", "separate"])
def test_config1_medium_full_state_all_rounds(layout):
    _need_gpu()
    _run_full(W.get(1), layout, drift_each_round=True)


def test_config1_medium_unpadded_stride():
    _need_gpu()
    w = W.get(1)
    _run_full(dataclasses.replace(w, rounds=3), "separate", stride=W.n_params(w))


def _run_per_tile(w, layout, stride=None, rounds=None):
    """Full-size run on the GPU in the launch configuration the benchmark times; the oracle
    replays all rounds on element columns that reach into EVERY tile of the fused kernel (one
    seeded element per tile) plus the first and last 4 elements of every component, i.e. every
    16-byte column that a component edge cuts (element columns never interact).  Compared after
    the first round (forward sweep), the second (backward sweep) and the last."""
    rounds = w.rounds if rounds is None else rounds
    off = W.component_offsets(w)
    P = int(off[-1])
    m = len(off) - 1
    pl = B.Plan(off, w.K, w.q, w.p, seed=w.seed)
    st = W.init_state(w, DEV, layout=layout, stride=stride, plan=pl)
    T = pl.info.tile_columns_blocked if layout == "blocked" else pl.info.tile_columns
    cols, red_off = W.tile_columns(off, 4 * T, seed=w.seed)
    n_tiles = pl.info.n_tiles if T == pl.info.tile_columns else None
    assert n_tiles is None or cols.size >= n_tiles
    idx = torch.from_numpy(cols).to(DEV)
    host = [st.gather(a, idx).cpu().numpy().copy() for a in range(3)]
    pads = [st.padding(a).clone() for a in range(3)]
    nbr = torch.zeros((m, w.K, w.q), dtype=torch.int32, device=DEV)
    compared = 0
    for r in range(rounds):
        _sync(pl, st, w, r)
        oracle.sync(red_off, w.K, pl.info.p, w.q, w.seed, r, *host, np.float32(w.eta), np.float32(w.zeta), w.mode)
        if r in (0, rounds - 1):
            pl.neighbours_device(r, nbr, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert (nbr.cpu().numpy() == oracle.neighbour_table(m, w.K, pl.info.p, w.q, w.seed, r)).all()
        if r in (0, 1, rounds - 1):
            for a, name in enumerate(("theta", "omega", "delta")):
                got = st.gather(a, idx).cpu().numpy()
                np.testing.assert_allclose(got, host[a], rtol=RTOL, atol=ATOL, err_msg=f"{w.name} {name} round {r}")
                assert (got == host[a]).all(), f"{w.name} {name} round {r}: {(got != host[a]).sum()} differ in the last bits"
                compared += got.size
    for a in range(3):
        assert torch.equal(st.padding(a), pads[a]), "padding was touched"
    # a property that holds at any size: with zeta = 1 in the paper's mode omega' is the
    # neighbour average, so the state stays bounded by the spread of the initial models
    for k in range(0, w.K, max(1, w.K // 4)):
        row = st.get_row(0, k)
        assert bool(torch.isfinite(row).all()) and float(row.abs().max()) < 10.0
    pl.destroy()
    print(f"{w.name} [{layout}]: {cols.size} element columns x {w.K} workers, {compared} values compared, all bit-equal")


def test_config2_large_vocab_every_tile_blocked():
    _need_gpu()
    _run_per_tile(W.get(2), "blocked")


def test_config2_large_vocab_every_tile_rows():
    _need_gpu()
    _run_per_tile(W.get(2), "rows", rounds=4)


def test_config2_large_vocab_unpadded_stride_takes_the_4_byte_path():
    _need_gpu()
    w = W.get(2)
    _run_per_tile(w, "separate", stride=W.n_params(w), rounds=2)


def test_config3_chunked_every_tile_blocked():
    _need_gpu()
    _run_per_tile(W.get(3), "blocked")


def test_config3_chunked_separate_tensors():
    _need_gpu()
    _run_per_tile(W.get(3), "separate", rounds=3)


def test_config4_k64_every_tile_blocked():
    _need_gpu()
    _run_per_tile(W.get(4), "blocked")


def test_config4_k64_every_tile_rows():
    _need_gpu()
    _run_per_tile(W.get(4), "rows", rounds=3)


def test_config4b_k64_4layer_every_tile_blocked():
    _need_gpu()
    _run_per_tile(W.get("k64_4layer"), "blocked")


@pytest.mark.parametrize("layout", ["blocked", "separate"])
def test_worker_rows_longer_than_2_to_31_elements(layout):
    # element offsets beyond 2^31 inside ONE worker row: every index in the kernels is 64-bit.
    # K = 4 workers of 2^31 + 70,003 parameters (103 GB of state); the oracle replays the rounds on
    # an element of every 97th tile, the edges of every component and the last 5000 elements.
    _need_gpu()
    K, q = 4, 1
    P = 2**31 + 70003
    off = np.array([0, 1000, 2**30 + 5, 2**31 - 3, 2**31 + 11, P], dtype=np.int64)
    pl = B.Plan(off, K, q, 0, seed=12)
    st = W.DeviceState(K, P, DEV, layout, plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(1)
    for buf in ([st.arena] if st.arena is not None else st.arrays):
        buf.normal_(0, 0.05, generator=g)
    T = pl.info.tile_columns_blocked if layout == "blocked" else pl.info.tile_columns
    cols, _ = W.tile_columns(off, 4 * T * 97, seed=3)
    cols = np.unique(np.concatenate([cols, np.arange(P - 5000, P, dtype=np.int64)]))
    red = np.searchsorted(cols, off).astype(np.int64)                # component boundaries among the sampled columns
    assert cols[-1] == P - 1 and (cols > 2**31).sum() > 5000
    idx = torch.from_numpy(cols).to(DEV)
    host = [st.gather(a, idx).cpu().numpy().copy() for a in range(3)]
    for r in range(3):
        if layout == "separate":
            pl.sync(*st.arrays, st.worker_stride, 0.9, 1.0, B.MODE_PAPER, r, None)
        else:
            pl.sync_state(st.desc(), 0.9, 1.0, B.MODE_PAPER, r, None)
        oracle.sync(red, K, pl.info.p, q, 12, r, *host, np.float32(0.9), np.float32(1.0), 1)
    torch.cuda.synchronize()
    for a, name in enumerate(("theta", "omega", "delta")):
        got = st.gather(a, idx).cpu().numpy()
        assert (got == host[a]).all(), f"{name}: {(got != host[a]).sum()} of {got.size} sampled values differ"
    out = torch.empty(P, device=DEV)
    if layout == "separate":
        pl.final_average(st.arrays[0], st.worker_stride, out, None)
    else:
        pl.final_average_state(st.desc(gossip_ma=True), out, None)
    torch.cuda.synchronize()
    assert (out.index_select(0, idx).cpu().numpy() == oracle.final_average(np.ascontiguousarray(host[0]))).all()
    pl.destroy()
