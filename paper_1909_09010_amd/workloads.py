"""Seeded synthetic workloads: LSTM-language-model-shaped parameter sets, their component
partitions and initial worker states.

This module holds shapes, sizes and value distributions only -- none of the method's
arithmetic -- and is the one module that both the HIP path's callers and the oracle's
callers (tests, bench) share.  The sync step never sees tokens, so the parameter sets
stand in for the paper's language models: ``large_vocab`` takes wiki-text-103's vocabulary
size (267,735, Section 3.1) and the paper's embedding width 512 (Section 3.2); eta = 0.9 and
zeta = 1.0 are the paper's BMUF settings (Section 3.2); (K, q) = (4, 1) and (8, 2) are its
4- and 8-GPU gossip settings (Section 3.3).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    K: int                      # workers
    q: int                      # neighbours drawn per component and sync
    vocab: int
    embed: int
    hidden: int
    layers: int
    chunk_rows: Optional[int]   # None: one component per tensor; else row chunks of every matrix
    eta: float
    zeta: float
    mode: int                   # 1 = Algorithm 1 as printed (Nesterov restart)
    rounds: int
    w0_dist: str                # "normal" or "uniform"
    w0_scale: float             # std, or half-width of U(-a, a)
    drift_std: float            # per-worker N(0, std) added to W0: stands for the local steps
    delta_std: float            # Delta init std (0 = zeros)
    seed: int
    p: int = 0                  # 0 = paper's rule p = log2(K) - 1
    kind: str = "lstm_lm"       # "lstm_lm": plain LSTM LM with full softmax; "paper": Section 3.2's model


# The five benchmark configurations (index = position in the benchmark's list) and "4b",
# the 4-layer variant whose size matches the "~135M params / ~104 GB" that config 4 states.
WORKLOADS = {
    "tiny": Workload("tiny", 4, 1, 1000, 64, 64, 2, None, 0.9, 1.0, 1, 10, "normal", 0.05, 0.01, 0.0, 0),
    "medium": Workload("medium", 8, 2, 10000, 650, 650, 2, None, 0.9, 1.0, 1, 50, "uniform", 0.05, 0.02, 0.0, 1),
    "large_vocab": Workload("large_vocab", 16, 3, 267735, 512, 512, 2, None, 0.875, 1.0, 1, 20,
                            "normal", 0.02, 0.005, 0.0, 2),
    "large_vocab_chunked": Workload("large_vocab_chunked", 16, 3, 267735, 512, 512, 2, 256, 0.9, 1.0, 1, 20,
                                    "normal", 0.02, 0.005, 0.0, 3),
    "k64": Workload("k64", 64, 4, 50000, 1024, 1024, 2, 1024, 0.95, 1.0, 1, 10, "normal", 0.02, 0.01, 1e-4, 4),
    "k64_4layer": Workload("k64_4layer", 64, 4, 50000, 1024, 1024, 4, 1024, 0.95, 1.0, 1, 10,
                           "normal", 0.02, 0.01, 1e-4, 4),
}
# The paper's own model and partition (Section 3.2): embedding 512 in 8 even shards, one LSTMP
# layer 2048/512 (LSTM weights one group, projection weights another), adaptive softmax with a
# head of 8192 words and 5 tails (projection factor 2), each tail its own group: 16 components;
# 16 workers with (p, q) = (3, 2) and sync periods (16, 128) (Section 3.3).  Tail sizes are not
# given in the paper; the remaining 259,543 words are split 16384/32768/49152/65536/95703.
WORKLOADS["paper_shaped"] = Workload("paper_shaped", 16, 2, 267735, 512, 2048, 1, None, 0.9, 1.0, 1, 16,
                                     "normal", 0.02, 0.005, 0.0, 5, 3, "paper")
PAPER_TAILS = (16384, 32768, 49152, 65536, 95703)
PAPER_HEAD = 8192
PAPER_PROJ = 512

CONFIG_ORDER = ["tiny", "medium", "large_vocab", "large_vocab_chunked", "k64"]


def get(name_or_index) -> Workload:
    if isinstance(name_or_index, int) or str(name_or_index).isdigit():
        return WORKLOADS[CONFIG_ORDER[int(name_or_index)]]
    return WORKLOADS[str(name_or_index)]


def scaled(w: Workload, vocab: int) -> Workload:
    """Same workload with a smaller vocabulary (parity tests at sizes the oracle finishes fast)."""
    return replace(w, name=f"{w.name}_v{vocab}", vocab=vocab)


def tensors(w: Workload) -> List[Tuple[str, int, int]]:
    """(name, rows, cols) of the flat parameter vector, in order.  cols = 1 for vectors."""
    if w.kind == "paper":
        out = [("embedding", w.vocab, w.embed),
               ("lstm.W+b", (w.embed + PAPER_PROJ) * 4 * w.hidden + 4 * w.hidden, 1),
               ("lstmp.projection", w.hidden, PAPER_PROJ),
               ("asm.head", PAPER_PROJ, PAPER_HEAD + len(PAPER_TAILS))]
        for i, n in enumerate(PAPER_TAILS, start=1):
            d = PAPER_PROJ >> i
            out.append((f"asm.tail{i}", PAPER_PROJ * d + d * n, 1))
        assert PAPER_HEAD + sum(PAPER_TAILS) == w.vocab
        return out
    out = [("embedding", w.vocab, w.embed)]
    for layer in range(w.layers):
        n_in = w.embed if layer == 0 else w.hidden
        out += [(f"lstm{layer}.W_ih", 4 * w.hidden, n_in), (f"lstm{layer}.W_hh", 4 * w.hidden, w.hidden),
                (f"lstm{layer}.bias", 4 * w.hidden, 1)]
    out += [("softmax.W", w.vocab, w.hidden), ("softmax.b", w.vocab, 1)]
    return out


def component_offsets(w: Workload) -> np.ndarray:
    """Element offsets of the components (m+1 entries).  Matrices are cut into chunks of
    ``chunk_rows`` rows when set; vectors stay whole."""
    sizes: List[int] = []
    if w.kind == "paper":
        for name, rows, cols in tensors(w):
            if name == "embedding":
                assert rows * cols % 8 == 0
                sizes += [rows * cols // 8] * 8
            else:
                sizes.append(rows * cols)
        return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))]).astype(np.int64)
    for _, rows, cols in tensors(w):
        if w.chunk_rows is None or cols == 1:
            sizes.append(rows * cols)
        else:
            for r0 in range(0, rows, w.chunk_rows):
                sizes.append((min(rows, r0 + w.chunk_rows) - r0) * cols)
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))]).astype(np.int64)


def periods(w: Workload) -> Optional[np.ndarray]:
    """Per-component sync periods H_i, or None when every component syncs at every call.
    The paper-shaped workload uses Section 3.3's (16, 128): embedding shards 128, others 16."""
    if w.kind != "paper":
        return None
    m = len(component_offsets(w)) - 1
    h = np.full(m, 16, dtype=np.int32)
    h[:8] = 128
    return h


def n_params(w: Workload) -> int:
    return int(sum(r * c for _, r, c in tensors(w)))


def padded_stride(P: int, multiple: int = 1024) -> int:
    return (P + multiple - 1) // multiple * multiple


class DeviceState:
    """theta, omega, delta of K workers on a device, in one of three placements, plus the
    plumbing tests and benchmarks need to move values in and out (no arithmetic of the method).

    layout "blocked": ONE arena [block][theta|omega|delta][worker][B floats]  (the library's
                      recommended placement, gbmuf_recommend_layout)
    layout "rows":    ONE arena [worker][theta|omega|delta][row padded to 4 KB]
    layout "separate": three separate [K, stride] tensors (stride = P padded to 4 KB unless given)
    """

    def __init__(self, K: int, P: int, device, layout: str = "blocked", stride: Optional[int] = None, plan=None):
        from . import binding
        self.K, self.P, self.layout = K, P, layout
        dev = torch.device(device)
        self.block_floats = self.block_stride = 0
        if layout == "separate":
            Pp = padded_stride(P) if stride is None else stride
            assert Pp >= P
            self.arena = None
            self.arrays = [torch.empty((K, Pp), device=dev, dtype=torch.float32) for _ in range(3)]
            self.worker_stride = Pp
            self.width = Pp
        else:
            assert stride is None
            kind = binding.LAYOUT_BLOCKED if layout == "blocked" else binding.LAYOUT_ROWS
            lay = binding.recommend_layout(P, K, kind, plan)
            self.arena = torch.empty(max(lay.arena_floats, 1), device=dev, dtype=torch.float32)
            self.worker_stride = lay.worker_stride
            self.block_floats, self.block_stride = lay.block_floats, lay.block_stride
            offs = (0, lay.omega_offset, lay.delta_offset)
            if layout == "rows":
                self.width = lay.omega_offset                       # the padded row
                self.arrays = [torch.as_strided(self.arena, (K, self.width), (lay.worker_stride, 1), o) for o in offs]
            else:
                B = lay.block_floats
                nb = (P + B - 1) // B
                self.width = nb * B
                # [K, nb, B] views: element (w, g, r) of array a sits at g*block_stride + a's offset + w*B + r
                self.arrays = [torch.as_strided(self.arena, (K, nb, B), (lay.worker_stride, lay.block_stride, 1), o)
                               for o in offs]

    # -- what the library is given --------------------------------------------------------
    def desc(self, gossip_ma: bool = False):
        from . import binding
        t, o, d = self.arrays
        return binding.make_state(t, None if gossip_ma else o, None if gossip_ma else d, self.worker_stride,
                                  self.block_floats, self.block_stride)

    @property
    def bytes(self) -> int:
        return 4 * (self.arena.numel() if self.arena is not None else sum(a.numel() for a in self.arrays))

    # -- moving values ----------------------------------------------------------------------
    def view2d(self, which: int) -> torch.Tensor:
        """[K, width] strided view for rows/separate; for blocked a [K, nb, B] view."""
        return self.arrays[which]

    def zero_(self):
        if self.arena is not None:
            self.arena.zero_()
        else:
            for a in self.arrays:
                a.zero_()

    def set_row(self, which: int, k: int, src: torch.Tensor) -> None:
        """worker k's first len(src) parameters of array `which` <- src (1-D, device)."""
        n = src.numel()
        a = self.arrays[which]
        if self.layout != "blocked":
            a[k, :n] = src
            return
        B = self.block_floats
        full = n // B
        if full:
            a[k, :full] = src[: full * B].view(full, B)
        if n % B:
            a[k, full, : n % B] = src[full * B:]

    def get_row(self, which: int, k: int) -> torch.Tensor:
        """worker k's P parameters of array `which` as a contiguous 1-D copy."""
        a = self.arrays[which]
        if self.layout != "blocked":
            return a[k, : self.P].clone()
        return a[k].reshape(-1)[: self.P].clone()

    def add_to_row(self, which: int, k: int, src: torch.Tensor) -> None:
        self.set_row(which, k, self.get_row(which, k)[: src.numel()] + src)

    def gather(self, which: int, cols: torch.Tensor) -> torch.Tensor:
        """[K, len(cols)] values of the given element columns (int64 device tensor)."""
        a = self.arrays[which]
        if self.layout != "blocked":
            return a.index_select(1, cols)
        B = self.block_floats
        return a[:, cols // B, cols % B]

    def padding(self, which: int) -> torch.Tensor:
        """The floats of array `which` beyond the P parameters (never touched by the library)."""
        a = self.arrays[which]
        if self.layout != "blocked":
            return a[:, self.P:]
        B = self.block_floats
        r = self.P % B
        return a[:, -1, r:] if r else a[:, :0, 0]

    def to_host(self, which: int):
        """[K, P] numpy copy."""
        import numpy as _np
        if self.layout != "blocked":
            return self.arrays[which][:, : self.P].cpu().numpy().copy()
        out = _np.empty((self.K, self.P), dtype=_np.float32)
        for k in range(self.K):
            out[k] = self.get_row(which, k).cpu().numpy()
        return out


def init_state(w: Workload, device, layout: str = "blocked", stride: Optional[int] = None, seed: Optional[int] = None,
               plan=None) -> DeviceState:
    """Seeded initial state of workload ``w``: W0 ~ w0_dist; theta_k = W0 + N(0, drift_std);
    omega_k = W0; Delta ~ N(0, delta_std) or 0.  Everything beyond the P parameters is zero.
    Generated row by row to bound temporary memory; the values do not depend on the layout."""
    P = n_params(w)
    dev = torch.device(device)
    st = DeviceState(w.K, P, dev, layout, stride=stride, plan=plan)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed if seed is None else seed)
    if w.w0_dist == "normal":
        w0 = torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.w0_scale
    else:
        w0 = (torch.rand(P, generator=g, device=dev, dtype=torch.float32) * 2 - 1) * w.w0_scale
    st.zero_()
    for k in range(w.K):
        st.set_row(1, k, w0)
        st.set_row(0, k, w0 + torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.drift_std)
        if w.delta_std > 0:
            st.set_row(2, k, torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.delta_std)
    return st


def drift_row(w: Workload, device, P: int, round: int, k: int) -> torch.Tensor:
    """Fresh seeded N(0, drift_std) noise for worker k's P parameters: the local training
    steps between two syncs."""
    g = torch.Generator(device=torch.device(device))
    g.manual_seed((1_000_003 * (w.seed + 1) + round) * 1024 + k)
    return torch.randn(P, generator=g, device=torch.device(device), dtype=torch.float32) * w.drift_std


def sample_columns(off: np.ndarray, edge: int = 48, interior: int = 32, seed: int = 0) -> np.ndarray:
    """Element columns for checking a large state against the oracle stripe by stripe: the
    first and last ``edge`` elements of every component plus ``interior`` random ones.
    Returns (columns ascending, reduced offsets) so that component indices are preserved."""
    rng = np.random.default_rng(seed)
    cols: List[np.ndarray] = []
    red = [0]
    for i in range(len(off) - 1):
        a, b = int(off[i]), int(off[i + 1])
        n = b - a
        if n <= 2 * edge + interior:
            pick = np.arange(a, b, dtype=np.int64)
        else:
            mid = rng.choice(n - 2 * edge, size=interior, replace=False) + a + edge
            pick = np.unique(np.concatenate([np.arange(a, a + edge), np.arange(b - edge, b), mid])).astype(np.int64)
        cols.append(pick)
        red.append(red[-1] + pick.size)
    return np.concatenate(cols) if cols else np.zeros(0, np.int64), np.asarray(red, dtype=np.int64)


def tile_columns(off: np.ndarray, tile_floats: int, seed: int = 0, edge: int = 4) -> Tuple[np.ndarray, np.ndarray]:
    """Element columns that reach into EVERY tile of a sync: tiles are the stretches of
    ``tile_floats`` elements between multiples of ``tile_floats`` (counted from the row start),
    cut at component boundaries.  One seeded element per (tile, component) piece, plus the
    first and last ``edge`` elements of every component (the 16-byte columns a component edge
    cuts).  Returns (columns ascending, reduced offsets) like ``sample_columns``."""
    rng = np.random.default_rng(seed)
    cols: List[np.ndarray] = []
    red = [0]
    for i in range(len(off) - 1):
        a, b = int(off[i]), int(off[i + 1])
        if b <= a:
            red.append(red[-1])
            continue
        t0, t1 = a // tile_floats, (b - 1) // tile_floats
        starts = np.arange(t0, t1 + 1, dtype=np.int64) * tile_floats
        lo = np.maximum(starts, a)
        hi = np.minimum(starts + tile_floats, b)
        pick = lo + (rng.random(lo.size) * (hi - lo)).astype(np.int64)
        ends = np.concatenate([np.arange(a, min(a + edge, b)), np.arange(max(b - edge, a), b)])
        pick = np.unique(np.concatenate([pick, ends])).astype(np.int64)
        cols.append(pick)
        red.append(red[-1] + pick.size)
    return (np.concatenate(cols) if cols else np.zeros(0, np.int64)), np.asarray(red, dtype=np.int64)
