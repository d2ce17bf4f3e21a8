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


def alloc_state(K: int, P: int, device, span_bytes: Optional[int] = None, stride: Optional[int] = None):
    """Uninitialised theta, omega, delta as [K, P_padded] float32 views plus their row stride.

    span_bytes None: three separate contiguous tensors (row stride = ``stride`` or P rounded
    up to 1024 floats = 4 KB, so that every row starts on a 4 KB boundary).  span_bytes set: ONE arena in which worker w's three rows sit side by side,
    [theta_w | omega_w | delta_w | gap], with the row stride chosen so that the K rows cover
    about span_bytes of HBM.  On MI355X the sync kernel is measurably faster when the rows it
    streams concurrently are spread over much more than ~70 GB of HBM address space (more
    independent DRAM banks); 150 GB is a good span for every benchmark configuration.
    """
    dev = torch.device(device)
    Pp = padded_stride(P) if stride is None else stride
    assert Pp >= P
    if span_bytes is None:
        return [torch.empty((K, Pp), device=dev, dtype=torch.float32) for _ in range(3)] + [Pp]
    assert stride is None
    from . import binding                       # the layout rule lives in the library
    lay = binding.recommend_layout(P, K, int(span_bytes))
    arena = torch.empty(lay.arena_floats, device=dev, dtype=torch.float32)
    S = lay.worker_stride
    views = [torch.as_strided(arena, (K, Pp), (S, 1), o) for o in (0, lay.omega_offset, lay.delta_offset)]
    return views + [S]


def default_span_bytes(device, state_bytes: int, want: int = 150 * 10**9) -> Optional[int]:
    """HBM span for alloc_state: ``want`` if it fits beside 8 GB of head room, else whatever
    does; None (contiguous layout) if the state itself is larger than that."""
    free, _ = torch.cuda.mem_get_info(torch.device(device))
    span = min(want, free - 8 * 10**9)
    return int(span) if span > state_bytes else None


def init_state(w: Workload, device, stride: Optional[int] = None, seed: Optional[int] = None,
               span_bytes: Optional[int] = None):
    """theta, omega, delta as [K, P_padded] float32 tensors (or strided views, see alloc_state)
    on ``device``; the row stride is ``theta.stride(0)``.
    W0 ~ w0_dist; theta_k = W0 + N(0, drift_std); omega_k = W0; Delta ~ N(0, delta_std) or 0.
    Padding columns (>= P) are zero.  Generated row by row to bound temporary memory."""
    P = n_params(w)
    dev = torch.device(device)
    theta, omega, delta, _ = alloc_state(w.K, P, dev, span_bytes=span_bytes, stride=stride)
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed if seed is None else seed)
    if w.w0_dist == "normal":
        w0 = torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.w0_scale
    else:
        w0 = (torch.rand(P, generator=g, device=dev, dtype=torch.float32) * 2 - 1) * w.w0_scale
    for t in (theta, omega, delta):
        t.zero_()
    for k in range(w.K):
        omega[k, :P] = w0
        theta[k, :P] = w0 + torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.drift_std
        if w.delta_std > 0:
            delta[k, :P] = torch.randn(P, generator=g, device=dev, dtype=torch.float32) * w.delta_std
    return theta, omega, delta


def drift(w: Workload, like: torch.Tensor, P: int, round: int) -> torch.Tensor:
    """Fresh seeded N(0, drift_std) noise of theta's shape (zero in the padding): the local
    training steps between two syncs."""
    g = torch.Generator(device=like.device)
    g.manual_seed(1_000_003 * (w.seed + 1) + round)
    out = torch.zeros_like(like)
    out[:, :P] = torch.randn((like.shape[0], P), generator=g, device=like.device, dtype=torch.float32) * w.drift_std
    return out


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
