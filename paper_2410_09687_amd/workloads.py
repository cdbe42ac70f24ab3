"""Seeded synthetic inputs for the MoIN hot path.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic (no distances, no matrix products) and is imported by both
the HIP-side callers and the oracle-side tests.

The paper's own workloads (SlimPajama documents, lm-eval-harness queries) are
not available; these inputs take their shapes and structure from the paper --
K = 5000 topics, rank-128 adapters on the 2048-wide TinyLlama projections
(Section 4 "Implementation details"), and expert usage concentrated on a small
share of the adapters (Table 3), modelled by Zipf draws -- and stand in for
them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20241009


@dataclass
class LinearWorkload:
    """One routed-LoRA projection: y[T,d_out] from x[T,d_in]."""
    name: str
    d_in: int
    d_out: int
    r: int
    E: int
    seq_lens: List[int]
    id_dist: str = "uniform"       # "uniform" | "zipf"
    zipf_s: float = 1.1
    scale: float = 2.0
    seed: int = BASE_SEED

    @property
    def S(self) -> int:
        return len(self.seq_lens)

    @property
    def T(self) -> int:
        return int(sum(self.seq_lens))

    def flops(self) -> float:
        """Algorithmic flops: base GEMM + shrink + expand, no padding or recompute."""
        return 2.0 * self.T * self.d_in * self.d_out + 2.0 * self.T * self.r * (self.d_in + self.d_out)


@dataclass
class RouteWorkload:
    name: str
    N: int
    K: int
    D: int
    dtype: str = "bf16"            # "bf16" | "f32"
    normalise: bool = True
    seed: int = BASE_SEED

    def flops(self) -> float:
        return 2.0 * self.N * self.K * self.D


# The five named configurations.
def config_tiny() -> Tuple[RouteWorkload, LinearWorkload]:
    return (RouteWorkload("c0_route", N=4, K=8, D=256, dtype="f32", normalise=False, seed=BASE_SEED),
            LinearWorkload("c0_tiny", 256, 256, 16, 8, [64] * 4, "uniform", scale=2.0, seed=BASE_SEED))


def config_prefill() -> LinearWorkload:
    return LinearWorkload("c1_q_proj_prefill", 2048, 2048, 64, 500, [512] * 64, "uniform",
                          scale=2.0, seed=BASE_SEED + 1)


def config_decode() -> List[LinearWorkload]:
    mk = lambda n, di, do, k: LinearWorkload(n, di, do, 128, 5000, [1] * 256, "zipf", 1.1, 2.0,
                                             BASE_SEED + 2 + 16 * k)
    return [mk("c2_gate_decode", 2048, 5632, 0), mk("c2_up_decode", 2048, 5632, 1),
            mk("c2_down_decode", 5632, 2048, 2)]


def config_router() -> RouteWorkload:
    return RouteWorkload("c3_router", N=1 << 20, K=5000, D=768, dtype="bf16", normalise=True,
                         seed=BASE_SEED + 3)


LAYER_PROJECTIONS = [  # name, d_in, d_out ; TinyLlama-shaped layer
    ("q", 2048, 2048), ("k", 2048, 256), ("v", 2048, 256), ("o", 2048, 2048),
    ("gate", 2048, 5632), ("up", 2048, 5632), ("down", 5632, 2048)]


def config_layer(seq_len: int = 2048, n_seq: int = 32, E: int = 5000, r: int = 128) -> List[LinearWorkload]:
    return [LinearWorkload(f"c4_{n}", di, do, r, E, [seq_len] * n_seq, "zipf", 1.5, 2.0,
                           BASE_SEED + 4 + 16 * i)
            for i, (n, di, do) in enumerate(LAYER_PROJECTIONS)]


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_bf16(shape, std: float, device, seed: int, chunk_elems: int = 1 << 28) -> torch.Tensor:
    """N(0, std^2) rounded to bf16, drawn in slabs so no fp32 copy of a huge
    stack is ever alive."""
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    g = _gen(device, seed)
    n = flat.numel()
    pos = 0
    while pos < n:
        m = min(chunk_elems, n - pos)
        tmp = torch.randn(m, generator=g, device=device, dtype=torch.float32)
        flat[pos:pos + m] = (tmp * std).to(torch.bfloat16)
        pos += m
    return out


def zipf_probabilities(E: int, s: float) -> np.ndarray:
    """p(rank k) proportional to k^-s for k = 1..E, truncated and normalised."""
    w = np.arange(1, E + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def draw_expert_ids(S: int, E: int, dist: str, zipf_s: float, seed: int, perm_seed=None) -> np.ndarray:
    """One expert id per sequence.  Zipf ranks are sent through a seeded
    permutation so popular experts are not neighbours in memory; batches of one
    request stream share ``perm_seed`` (the same experts stay popular)."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        return rng.integers(0, E, size=S, dtype=np.int64).astype(np.int32)
    if dist == "zipf":
        ranks = rng.choice(E, size=S, p=zipf_probabilities(E, zipf_s))
        perm = np.random.default_rng((seed ^ 0x5EED) if perm_seed is None else perm_seed).permutation(E)
        return perm[ranks].astype(np.int32)
    raise ValueError(f"unknown id distribution {dist!r}")


def seq_offsets_of(seq_lens) -> np.ndarray:
    off = np.zeros(len(seq_lens) + 1, dtype=np.int64)
    np.cumsum(np.asarray(seq_lens, dtype=np.int64), out=off[1:])
    if off[-1] >= 2 ** 31:
        raise ValueError("token count does not fit int32 offsets")
    return off.astype(np.int32)


@dataclass
class LinearInputs:
    wl: LinearWorkload
    x: torch.Tensor            # [T, d_in] bf16
    W: torch.Tensor            # [d_out, d_in] bf16
    A_stack: torch.Tensor      # [E, r, d_in] bf16
    B_stack: torch.Tensor      # [E, d_out, r] bf16
    seq_offsets: torch.Tensor  # [S+1] int32
    expert_ids: torch.Tensor   # [S] int32
    extra: dict = field(default_factory=dict)


def make_linear_inputs(wl: LinearWorkload, device="cpu", expert_ids: Optional[np.ndarray] = None,
                       x: Optional[torch.Tensor] = None, stacks: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                       ) -> LinearInputs:
    """x ~ N(0,1); W, A_e ~ N(0, 1/d_in); B_e ~ N(0, 1/r); all rounded to bf16."""
    dev = torch.device(device)
    T = wl.T
    if x is None:
        x = _randn_bf16((T, wl.d_in), 1.0, dev, wl.seed * 8 + 0)
    W = _randn_bf16((wl.d_out, wl.d_in), wl.d_in ** -0.5, dev, wl.seed * 8 + 1)
    if stacks is None:
        A = _randn_bf16((wl.E, wl.r, wl.d_in), wl.d_in ** -0.5, dev, wl.seed * 8 + 2)
        B = _randn_bf16((wl.E, wl.d_out, wl.r), wl.r ** -0.5, dev, wl.seed * 8 + 3)
    else:
        A, B = stacks
    if expert_ids is None:
        expert_ids = draw_expert_ids(wl.S, wl.E, wl.id_dist, wl.zipf_s, wl.seed * 8 + 4)
    off = seq_offsets_of(wl.seq_lens)
    return LinearInputs(wl, x, W, A, B,
                        torch.from_numpy(off).to(dev),
                        torch.from_numpy(np.asarray(expert_ids, dtype=np.int32)).to(dev))


@dataclass
class RouteInputs:
    wl: RouteWorkload
    emb: torch.Tensor        # [N, D]
    centroids: torch.Tensor  # [K, D]


def _embeddings(n: int, D: int, dtype: str, normalise: bool, device, seed: int,
                chunk_rows: int = 1 << 18) -> torch.Tensor:
    """N(0,1) in fp32, optionally scaled to unit L2 length in fp32, then rounded
    to the storage type (so stored bf16 norms are close to, not exactly, 1)."""
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    out = torch.empty((n, D), dtype=tdt, device=device)
    g = _gen(device, seed)
    for lo in range(0, n, chunk_rows):
        hi = min(n, lo + chunk_rows)
        v = torch.randn((hi - lo, D), generator=g, device=device, dtype=torch.float32)
        if normalise:
            v = v / v.norm(dim=1, keepdim=True)
        out[lo:hi] = v.to(tdt)
    return out


def make_route_inputs(wl: RouteWorkload, device="cpu") -> RouteInputs:
    dev = torch.device(device)
    return RouteInputs(wl,
                       _embeddings(wl.N, wl.D, wl.dtype, wl.normalise, dev, wl.seed * 8 + 5),
                       _embeddings(wl.K, wl.D, wl.dtype, wl.normalise, dev, wl.seed * 8 + 6))


def retained_slot_table(K: int, keep: int, seed: int) -> np.ndarray:
    """slot_of_centroid[K]: `keep` seeded-random centroids get adapter slots
    0..keep-1 in index order, the rest -1 (clusters too small to train on)."""
    rng = np.random.default_rng(seed)
    kept = np.sort(rng.choice(K, size=keep, replace=False))
    table = np.full(K, -1, dtype=np.int32)
    table[kept] = np.arange(keep, dtype=np.int32)
    return table


# ---- host views for the oracle (bit patterns, never arithmetic) ---------------

def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16 tensor, on the host."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def compact_stacks(inp: LinearInputs):
    """Host copies of only the experts a batch references, with ids remapped to
    the compact numbering (a 5000-expert stack does not fit a test's host RAM)."""
    ids = inp.expert_ids.cpu().numpy().astype(np.int64)
    used = np.unique(ids[ids >= 0])
    remap = {int(e): i for i, e in enumerate(used)}
    new_ids = np.array([remap[int(e)] if e >= 0 else -1 for e in ids], dtype=np.int32)
    if used.size == 0:
        return None, None, new_ids
    sel = torch.from_numpy(used).to(inp.A_stack.device)
    A = bf16_bits(inp.A_stack.index_select(0, sel))
    B = bf16_bits(inp.B_stack.index_select(0, sel))
    return A, B, new_ids
