"""gbmuf_sync_static, the entry point for callers that cannot allocate: its neighbour table
lives in a static device array of the library instead of the plan's scratch.  Checked against
gbmuf_sync_state bit for bit, through the C ABI, on two calls in a row of which the second has
the smaller input (so stale rows of the first call lie beyond what the second one draws).
Collected last on purpose (file name): a failure here must not hide the other tests."""
import numpy as np
import pytest

from paper_1909_09010_amd import binding as B
from paper_1909_09010_amd import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _pair(K, q, sizes, periods=None, layout="blocked", seed=0, rounds=(0, 1, 2)):
    """Runs the same syncs through gbmuf_sync_state and gbmuf_sync_static on two copies of one
    seeded state and returns True if every float of the two arenas is equal."""
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    P = int(off[-1])
    pl = B.Plan(off, K, q, 0, seed=seed + 1, periods=periods)
    a = W.DeviceState(K, P, DEV, layout, plan=pl)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    a.arena.normal_(0, 0.05, generator=g)
    b = W.DeviceState(K, P, DEV, layout, plan=pl)
    b.arena.copy_(a.arena)
    initial = a.arena.clone()
    stream = torch.cuda.current_stream()
    for r in rounds:
        pl.sync_state(a.desc(), 0.9, 1.0, B.MODE_PAPER, r, stream)
        pl.sync_static(b.desc(), 0.9, 1.0, B.MODE_PAPER, r, stream)
    torch.cuda.synchronize()
    same = torch.equal(a.arena, b.arena)
    changed = not torch.equal(a.arena, initial)
    pl.destroy()
    return same and changed


def test_static_table_sync_equals_the_plan_scratch_sync_twice_in_a_row_second_call_smaller():
    _need_gpu()
    # first call: 300 components x 16 workers x q = 6 (28,800 table entries, several hundred tiles)
    assert _pair(16, 6, [4000 + 7 * i for i in range(300)], seed=1)
    # second call, right after, with a smaller input and a narrower table (5 x 8 x 2 = 80 entries)
    assert _pair(8, 2, [3000, 1, 4099, 0, 513], seed=2)
    # and once more in rows, with a different q per component and gossip-MA left to the other tests
    assert _pair(16, [3, 0, 6, 1], [2048, 33120, 35168, 50000], layout="rows", seed=3)


def test_static_table_sync_refuses_a_table_beyond_its_size():
    _need_gpu()
    m = B.STATIC_TABLE_ENTRIES // (64 * 4) + 1            # m * K * q just above the limit
    off = np.arange(m + 1, dtype=np.int64) * 8
    pl = B.Plan(off, 64, 4, 0, seed=0)
    st = W.DeviceState(64, int(off[-1]), DEV, "blocked", plan=pl)
    st.zero_()
    before = st.arena.clone()
    with pytest.raises(B.GbmufError) as e:
        pl.sync_static(st.desc(), 0.9, 1.0, B.MODE_PAPER, 0, None)
    assert e.value.code == B.GBMUF_EUNSUPPORTED and "static table" in str(e.value)
    pl.sync_state(st.desc(), 0.9, 1.0, B.MODE_PAPER, 0, None)     # the ordinary entry point still takes it
    torch.cuda.synchronize()
    assert torch.equal(st.arena, before)                            # all zeros stay zeros: a fixed point
    pl.destroy()


def test_static_table_sync_can_be_captured_in_a_hip_graph_and_replayed():
    # the call allocates nothing and never synchronises, so it is legal under stream capture; every
    # replay (with eager work and synchronisation between replays) must equal the eager calls
    _need_gpu()
    K, q = 16, 3
    off = np.concatenate([[0], np.cumsum([5000, 70001, 12, 9000])]).astype(np.int64)
    P = int(off[-1])
    pl = B.Plan(off, K, q, 0, seed=9)
    g = torch.Generator(device=DEV)
    g.manual_seed(4)
    graphed = W.DeviceState(K, P, DEV, "blocked", plan=pl)
    graphed.arena.normal_(0, 0.05, generator=g)
    eager = W.DeviceState(K, P, DEV, "blocked", plan=pl)
    eager.arena.copy_(graphed.arena)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for r in range(3):
            pl.sync_static(graphed.desc(), 0.9, 1.0, B.MODE_PAPER, r, torch.cuda.current_stream())
    for replay in range(3):
        graph.replay()
        for r in range(3):
            pl.sync_state(eager.desc(), 0.9, 1.0, B.MODE_PAPER, r, None)
        torch.cuda.synchronize()
        assert torch.equal(graphed.arena, eager.arena), f"replay {replay}"
        junk = torch.randn(1 << 20, device=DEV).sum().item()          # eager work between the replays
        assert junk == junk
    pl.destroy()
