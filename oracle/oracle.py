"""ctypes front end of ``moin_oracle.c`` (test infrastructure only).

Inputs are numpy arrays.  bf16 data travels as ``uint16`` bit patterns (numpy
has no bf16); fp32 as ``float32``.  Every result is fp64 / exact integer.
Nothing here touches a GPU or the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moin_oracle.c")
_LIB = os.path.join(_HERE, "libmoin_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64 arithmetic, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
               "-fno-fast-math", "-ffp-contract=off", _SRC, "-o", _LIB + ".tmp", "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.moin_oracle_dist2.argtypes = [c.c_void_p, c.c_void_p, c.c_int32, c.c_int,
                                          c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p]
        lib.moin_oracle_route.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                          c.c_int32, c.c_int, c.c_void_p, c.c_void_p,
                                          c.c_void_p, c.c_void_p]
        lib.moin_oracle_slot_map.argtypes = [c.c_void_p, c.c_int64, c.c_void_p, c.c_int32,
                                             c.c_void_p]
        lib.moin_oracle_histogram.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p]
        lib.moin_oracle_merge_adapters.argtypes = [c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
                                                   c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p]
        lib.moin_oracle_route_topk.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_int,
                                               c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p]
        lib.moin_oracle_lora_linear.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int64,
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
            c.c_double, c.c_void_p, c.c_int32, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p, c.c_int32]
        lib.moin_oracle_lora_linear_mx.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int64,
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
            c.c_int32, c.c_double, c.c_void_p, c.c_int32, c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p,
            c.c_int32]
        lib.moin_oracle_mx_quantize.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p,
                                                c.c_void_p]
        lib.moin_oracle_mx_dequantize.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int32,
                                                  c.c_void_p]
        lib.moin_oracle_kmeans_update.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_void_p,
                                                  c.c_int32, c.c_int32, c.c_int, c.c_void_p,
                                                  c.c_void_p, c.c_void_p]
        lib.moin_oracle_kmeans_update.restype = c.c_int
        lib.moin_oracle_retain_clusters.argtypes = [c.c_void_p, c.c_int32, c.c_int64, c.c_void_p]
        lib.moin_oracle_retain_clusters.restype = c.c_int
        for f in ("moin_oracle_dist2", "moin_oracle_route", "moin_oracle_slot_map",
                  "moin_oracle_histogram", "moin_oracle_lora_linear",
                  "moin_oracle_lora_linear_mx", "moin_oracle_mx_quantize",
                  "moin_oracle_mx_dequantize",
                  "moin_oracle_max_threads"):
            getattr(lib, f).restype = c.c_int
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _emb_array(a, name):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, 0
    if a.dtype == np.uint16:
        return a, 1
    raise TypeError(f"{name}: float32 or uint16 (bf16 bits) expected, got {a.dtype}")


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid argument (code {rc})")


def max_threads() -> int:
    return int(_load().moin_oracle_max_threads())


def route(emb, centroids, eligible=None, want_gaps=False):
    """argmin_k ||q_i - c_k||^2 per query; ties to the lowest k.

    Returns ``ids`` (int32 centroid indices), plus ``(best_d2, second_d2)`` in
    fp64 when ``want_gaps``.  ``eligible`` (bool[K]) limits the search.
    """
    emb, dt = _emb_array(emb, "emb")
    centroids, dt2 = _emb_array(centroids, "centroids")
    if dt != dt2 or emb.ndim != 2 or centroids.ndim != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] must share dtype and D")
    N, D = emb.shape
    K = centroids.shape[0]
    ids = np.zeros(N, dtype=np.int32)
    best = np.zeros(N, dtype=np.float64) if want_gaps else None
    second = np.zeros(N, dtype=np.float64) if want_gaps else None
    el = None
    if eligible is not None:
        el = np.ascontiguousarray(np.asarray(eligible).astype(np.uint8))
        if el.shape != (K,):
            raise ValueError("eligible must have shape [K]")
    _check(_load().moin_oracle_route(_ptr(emb), _ptr(centroids), N, K, D, dt, _ptr(el),
                                     _ptr(ids), _ptr(best), _ptr(second)), "route")
    return (ids, best, second) if want_gaps else ids


def route_topk(emb, centroids, k, eligible=None):
    """The k nearest centroids of every query, nearest first, equal distances by increasing index:
    ``(ids [N,k] int32, d2 [N,k] float64)``; -1 / inf where fewer than k centroids are eligible."""
    emb, dt = _emb_array(emb, "emb")
    centroids, dt2 = _emb_array(centroids, "centroids")
    if dt != dt2 or emb.ndim != 2 or centroids.ndim != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] must share dtype and D")
    if int(k) <= 0:
        raise ValueError("k must be positive")
    N, D = emb.shape
    K = centroids.shape[0]
    ids = np.zeros((N, int(k)), dtype=np.int32)
    d2 = np.zeros((N, int(k)), dtype=np.float64)
    el = None
    if eligible is not None:
        el = np.ascontiguousarray(np.asarray(eligible).astype(np.uint8))
        if el.shape != (K,):
            raise ValueError("eligible must have shape [K]")
    _check(_load().moin_oracle_route_topk(_ptr(emb), _ptr(centroids), N, K, D, dt, _ptr(el), int(k),
                                          _ptr(ids), _ptr(d2)), "route_topk")
    return ids, d2


def dist2(emb, centroids, qi, ki):
    """fp64 squared distances for the (query, centroid) pairs ``(qi[p], ki[p])``."""
    emb, dt = _emb_array(emb, "emb")
    centroids, dt2 = _emb_array(centroids, "centroids")
    if dt != dt2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("dtype / D mismatch")
    qi = np.ascontiguousarray(qi, dtype=np.int64)
    ki = np.ascontiguousarray(ki, dtype=np.int32)
    if qi.shape != ki.shape:
        raise ValueError("qi and ki must have the same shape")
    if qi.size and (qi.min() < 0 or qi.max() >= emb.shape[0] or ki.min() < 0
                    or ki.max() >= centroids.shape[0]):
        raise ValueError("pair index out of range")
    out = np.zeros(qi.shape, dtype=np.float64)
    _check(_load().moin_oracle_dist2(_ptr(emb), _ptr(centroids), emb.shape[1], dt, _ptr(qi),
                                     _ptr(ki), qi.size, _ptr(out)), "dist2")
    return out


def slot_map(centroid_ids, slot_of_centroid):
    centroid_ids = np.ascontiguousarray(centroid_ids, dtype=np.int32)
    slot_of_centroid = np.ascontiguousarray(slot_of_centroid, dtype=np.int32)
    out = np.zeros_like(centroid_ids)
    _check(_load().moin_oracle_slot_map(_ptr(centroid_ids), centroid_ids.size,
                                        _ptr(slot_of_centroid), slot_of_centroid.size,
                                        _ptr(out)), "slot_map")
    return out


def histogram(ids, K):
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    counts = np.zeros(K, dtype=np.int64)
    _check(_load().moin_oracle_histogram(_ptr(ids), ids.size, K, _ptr(counts)), "histogram")
    return counts


def kmeans_update(emb, ids, old_centroids):
    """Centre update of one Lloyd iteration (fp64): returns ``(new_centroids
    [K,D] float64, counts [K] int64, inertia float)``.  A centre with no
    members keeps its old value; inertia is measured against the old centres."""
    emb, dt = _emb_array(emb, "emb")
    old_centroids, dt2 = _emb_array(old_centroids, "old_centroids")
    if dt != dt2 or emb.ndim != 2 or old_centroids.ndim != 2 or emb.shape[1] != old_centroids.shape[1]:
        raise ValueError("emb [N,D] and old_centroids [K,D] must share dtype and D")
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    N, D = emb.shape
    K = old_centroids.shape[0]
    if ids.shape != (N,):
        raise ValueError("ids must have shape [N]")
    new_c = np.zeros((K, D), dtype=np.float64)
    counts = np.zeros(K, dtype=np.int64)
    inertia = np.zeros(1, dtype=np.float64)
    _check(_load().moin_oracle_kmeans_update(_ptr(emb), _ptr(ids), N, _ptr(old_centroids), K, D, dt,
                                             _ptr(new_c), _ptr(counts), _ptr(inertia)), "kmeans_update")
    return new_c, counts, float(inertia[0])


def retain_clusters(counts, min_count):
    """Adapter slot of each cluster (kept clusters numbered in ascending order,
    -1 for clusters with fewer than ``min_count`` members) and how many are kept."""
    counts = np.ascontiguousarray(counts, dtype=np.int64)
    slot = np.zeros(counts.size, dtype=np.int32)
    kept = _load().moin_oracle_retain_clusters(_ptr(counts), counts.size, int(min_count), _ptr(slot))
    if kept < 0:
        raise ValueError("oracle retain_clusters: invalid argument")
    return slot, int(kept)


ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "silu": 2, "gelu": 3}


def _activation_code(activation):
    if activation not in ACTIVATIONS:
        raise ValueError(f"activation: one of {sorted(k for k in ACTIVATIONS if k)} or None expected")
    return ACTIVATIONS[activation]


def lora_linear(x, seq_offsets, expert_ids, W, A_stack, B_stack, scale, rows=None,
                threads=None, rank_of_expert=None, activation=None):
    """y = x W^T + scale * act(x A_e^T) B_e^T with one expert per sequence (fp64);
    ``activation``: None (the paper's linear adapter), "relu", "silu" or "gelu"
    ("Future Works", better adapters: an activation between the two LoRA layers).

    ``x [T,d_in]``, ``W [d_out,d_in]``, ``A_stack [E,r,d_in]``, ``B_stack
    [E,d_out,r]`` are uint16 bf16 bit patterns.  ``rows`` selects the tokens to
    compute (default all); the result is ``[len(rows), d_out]`` float64.
    ``rank_of_expert [E]`` (optional): expert e uses only its first
    ``rank_of_expert[e]`` rows of A_e / columns of B_e.
    """
    x = np.ascontiguousarray(x)
    W = np.ascontiguousarray(W)
    for name, a in (("x", x), ("W", W)):
        if a.dtype != np.uint16 or a.ndim != 2:
            raise TypeError(f"{name}: 2-D uint16 (bf16 bits) expected")
    T, d_in = x.shape
    d_out = W.shape[0]
    if W.shape[1] != d_in:
        raise ValueError("W must be [d_out, d_in]")
    seq_offsets = np.ascontiguousarray(seq_offsets, dtype=np.int32)
    expert_ids = np.ascontiguousarray(expert_ids, dtype=np.int32)
    S = expert_ids.size
    if seq_offsets.size != S + 1:
        raise ValueError("seq_offsets must have S+1 entries")
    if A_stack is None or B_stack is None:
        E, r = 0, 0
        A_stack = B_stack = None
    else:
        A_stack = np.ascontiguousarray(A_stack)
        B_stack = np.ascontiguousarray(B_stack)
        if A_stack.dtype != np.uint16 or B_stack.dtype != np.uint16:
            raise TypeError("A_stack/B_stack: uint16 (bf16 bits) expected")
        E, r = A_stack.shape[0], A_stack.shape[1]
        if A_stack.shape != (E, r, d_in) or B_stack.shape != (E, d_out, r):
            raise ValueError("A_stack [E,r,d_in] / B_stack [E,d_out,r] shape mismatch")
    if rows is None:
        rows_arr, n_rows = None, T
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_rows = rows_arr.size
    ranks = None
    if rank_of_expert is not None:
        ranks = np.ascontiguousarray(rank_of_expert, dtype=np.int32)
        if ranks.shape != (E,):
            raise ValueError("rank_of_expert must have E entries")
    y = np.zeros((n_rows, d_out), dtype=np.float64)
    slots = int(threads) if threads else max_threads()
    work = np.zeros(slots * (d_in + max(r, 1)), dtype=np.float64)
    _check(_load().moin_oracle_lora_linear(
        _ptr(x), _ptr(seq_offsets), _ptr(expert_ids), S, T, _ptr(W), _ptr(A_stack),
        _ptr(B_stack), E, d_in, d_out, r, float(scale), _ptr(ranks), _activation_code(activation),
        _ptr(rows_arr), n_rows, _ptr(y), _ptr(work), slots), "lora_linear")
    return y


def merge_adapters(A_stack, B_stack, ids, weights, r_out):
    """One adapter of rank ``len(ids) * r`` (zero-padded to ``r_out``) that stands for
    ``sum_m weights[m] * B[ids[m]] @ A[ids[m]]`` ("Future Works", creating new experts on the fly):
    returns ``(A_out [r_out, d_in], B_out [d_out, r_out])`` as bf16 bit patterns."""
    A_stack = np.ascontiguousarray(A_stack)
    B_stack = np.ascontiguousarray(B_stack)
    if A_stack.dtype != np.uint16 or B_stack.dtype != np.uint16 or A_stack.ndim != 3 or B_stack.ndim != 3:
        raise TypeError("A_stack [E,r,d_in] / B_stack [E,d_out,r]: uint16 (bf16 bits) expected")
    E, r, d_in = A_stack.shape
    d_out = B_stack.shape[1]
    if B_stack.shape != (E, d_out, r):
        raise ValueError("A_stack [E,r,d_in] / B_stack [E,d_out,r] shape mismatch")
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    if ids.shape != weights.shape or ids.ndim != 1:
        raise ValueError("ids and weights: one entry per merged adapter")
    A_out = np.zeros((int(r_out), d_in), dtype=np.uint16)
    B_out = np.zeros((d_out, int(r_out)), dtype=np.uint16)
    _check(_load().moin_oracle_merge_adapters(_ptr(A_stack), _ptr(B_stack), E, r, d_in, d_out, _ptr(ids),
                                              _ptr(weights), ids.size, int(r_out), _ptr(A_out), _ptr(B_out)),
           "merge_adapters")
    return A_out, B_out


MX_BLOCK = 32


def mx_quantize(values):
    """MXFP8 quantisation along the last axis of ``values [rows, cols]`` (uint16
    bf16 bit patterns, finite, cols a multiple of 32): returns ``codes [rows,
    cols]`` (uint8 FP8 E4M3) and ``scales [rows, cols/32]`` (uint8 E8M0)."""
    v = np.ascontiguousarray(values)
    if v.dtype != np.uint16 or v.ndim != 2:
        raise TypeError("values: 2-D uint16 (bf16 bits) expected")
    rows, cols = v.shape
    if cols == 0 or cols % MX_BLOCK:
        raise ValueError("cols must be a positive multiple of 32")
    codes = np.zeros((rows, cols), dtype=np.uint8)
    scales = np.zeros((rows, cols // MX_BLOCK), dtype=np.uint8)
    _check(_load().moin_oracle_mx_quantize(_ptr(v), rows, cols, _ptr(codes), _ptr(scales)),
           "mx_quantize")
    return codes, scales


def mx_dequantize(codes, scales):
    """fp64 values of an MXFP8 matrix (exact)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    rows, cols = codes.shape
    if cols == 0 or cols % MX_BLOCK or scales.shape != (rows, cols // MX_BLOCK):
        raise ValueError("codes [rows, cols] / scales [rows, cols/32] shape mismatch")
    out = np.zeros((rows, cols), dtype=np.float64)
    _check(_load().moin_oracle_mx_dequantize(_ptr(codes), _ptr(scales), rows, cols, _ptr(out)),
           "mx_dequantize")
    return out


def lora_linear_mx(x, seq_offsets, expert_ids, Wq, Ws, A_stack, B_stack, scale, rows=None,
                   threads=None, rank_of_expert=None, activation=None):
    """Routed LoRA linear on an MXFP8 base: y = xd Wd^T + scale * (x A_e^T) B_e^T
    with Wd the dequantised weight (``Wq [d_out,d_in]`` codes, ``Ws
    [d_out,d_in/32]`` scales), xd the bf16 activations after an MXFP8 round trip
    and the adapter term on the bf16 activations themselves (fp64)."""
    x = np.ascontiguousarray(x)
    if x.dtype != np.uint16 or x.ndim != 2:
        raise TypeError("x: 2-D uint16 (bf16 bits) expected")
    Wq = np.ascontiguousarray(Wq)
    Ws = np.ascontiguousarray(Ws)
    if Wq.dtype != np.uint8 or Ws.dtype != np.uint8 or Wq.ndim != 2:
        raise TypeError("Wq / Ws: uint8 expected")
    T, d_in = x.shape
    d_out = Wq.shape[0]
    if d_in % MX_BLOCK or Wq.shape[1] != d_in or Ws.shape != (d_out, d_in // MX_BLOCK):
        raise ValueError("Wq [d_out, d_in] / Ws [d_out, d_in/32] shape mismatch")
    seq_offsets = np.ascontiguousarray(seq_offsets, dtype=np.int32)
    expert_ids = np.ascontiguousarray(expert_ids, dtype=np.int32)
    S = expert_ids.size
    if seq_offsets.size != S + 1:
        raise ValueError("seq_offsets must have S+1 entries")
    if A_stack is None or B_stack is None:
        E, r = 0, 0
        A_stack = B_stack = None
    else:
        A_stack = np.ascontiguousarray(A_stack)
        B_stack = np.ascontiguousarray(B_stack)
        if A_stack.dtype != np.uint16 or B_stack.dtype != np.uint16:
            raise TypeError("A_stack/B_stack: uint16 (bf16 bits) expected")
        E, r = A_stack.shape[0], A_stack.shape[1]
        if A_stack.shape != (E, r, d_in) or B_stack.shape != (E, d_out, r):
            raise ValueError("A_stack [E,r,d_in] / B_stack [E,d_out,r] shape mismatch")
    if rows is None:
        rows_arr, n_rows = None, T
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        n_rows = rows_arr.size
    ranks = None
    if rank_of_expert is not None:
        ranks = np.ascontiguousarray(rank_of_expert, dtype=np.int32)
        if ranks.shape != (E,):
            raise ValueError("rank_of_expert must have E entries")
    y = np.zeros((n_rows, d_out), dtype=np.float64)
    slots = int(threads) if threads else max_threads()
    work = np.zeros(slots * (2 * d_in + max(r, 1)), dtype=np.float64)
    _check(_load().moin_oracle_lora_linear_mx(
        _ptr(x), _ptr(seq_offsets), _ptr(expert_ids), S, T, _ptr(Wq), _ptr(Ws), _ptr(A_stack),
        _ptr(B_stack), E, d_in, d_out, r, float(scale), _ptr(ranks), _activation_code(activation),
        _ptr(rows_arr), n_rows, _ptr(y), _ptr(work), slots), "lora_linear_mx")
    return y


class AdapterCache:
    """Residency of adapters in a fixed number of GPU slots (Section 2, serving
    paragraph: adapters live in CPU memory, the most frequently routed ones are
    cached on the GPU).  Plain bookkeeping, one batch at a time:

    * each sequence adds one use to its expert;
    * an expert the batch needs is always brought in;
    * a free slot is taken lowest index first, otherwise the resident expert that
      the batch does not need with the fewest uses goes (then the one used
      longest ago, then the lowest slot);
    * with no such expert left the newcomer gets no slot (-1: base model only).

    protect_previous: a server that pages the adapters of batch k+1 in while batch k is
    still computing must not overwrite what batch k reads, so the experts of the batch
    admitted just before are as untouchable as the batch's own.
    """

    def __init__(self, n_experts, n_slots, protect_previous=False):
        self.protect_previous = bool(protect_previous)
        self.previous = []
        self.n_experts, self.n_slots = int(n_experts), int(n_slots)
        self.slot_of = {}                      # expert -> slot
        self.expert_in = [None] * self.n_slots
        self.uses = {}
        self.last = {}
        self.batches = 0
        self.hits = self.misses = self.loads = self.evictions = self.overflows = 0

    def admit(self, expert_ids):
        ids = [int(e) for e in expert_ids]
        if any(e < -1 or e >= self.n_experts for e in ids):
            raise ValueError("expert id out of range")
        self.batches += 1
        needed = []
        for e in ids:
            if e >= 0 and e not in needed:
                needed.append(e)
        for e in needed:
            self.uses[e] = self.uses.get(e, 0) + ids.count(e)
            self.last[e] = self.batches
        loaded = []
        for e in needed:
            n = ids.count(e)
            if e in self.slot_of:
                self.hits += n
                continue
            self.misses += n
            free = [s for s in range(self.n_slots) if self.expert_in[s] is None]
            if free:
                slot = free[0]
            else:
                keep = needed + (self.previous if self.protect_previous else [])
                cand = [s for s in range(self.n_slots) if self.expert_in[s] not in keep]
                if not cand:
                    self.overflows += 1
                    continue
                slot = min(cand, key=lambda s: (self.uses[self.expert_in[s]], self.last[self.expert_in[s]], s))
                del self.slot_of[self.expert_in[slot]]
                self.evictions += 1
            self.expert_in[slot] = e
            self.slot_of[e] = slot
            self.loads += 1
            loaded.append((e, slot))
        self.previous = needed
        slots = np.array([self.slot_of.get(e, -1) if e >= 0 else -1 for e in ids], dtype=np.int32)
        return slots, loaded

    def tables(self):
        slot_of = np.full(self.n_experts, -1, dtype=np.int32)
        for e, s in self.slot_of.items():
            slot_of[e] = s
        expert_in = np.array([-1 if e is None else e for e in self.expert_in], dtype=np.int32)
        return slot_of, expert_in
