"""Thin ctypes binding of ``libmoin.so`` -- argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current torch stream across the C ABI declared in
``include/moin.h`` and returns torch tensors.  No step of the method runs
here, and there is no fallback: without the built library, or with tensors
that are not on a GPU, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoin.so")

MOIN_F32, MOIN_BF16 = 0, 1
MOIN_MX_X_INTERNAL, MOIN_MX_X_EMIT, MOIN_MX_X_GIVEN = 0, 1, 2
MOIN_ROUTE_RETAINED_ONLY = 1
MOIN_ROUTE_SAME_CENTROIDS = 2
(K_PLAN, K_SHRINK, K_LINEAR, K_ROUTE, K_ROUTE_AUX, K_DECODE_SHRINK, K_DECODE_EXPAND, K_DECODE_BASE,
 K_KMEANS_SORT, K_KMEANS_SUM, K_KMEANS_FINAL) = range(11)
KERNEL_NAMES = ["plan", "shrink", "linear", "route", "route_aux", "decode_shrink", "decode_expand",
                "decode_base", "kmeans_sort", "kmeans_sum", "kmeans_final", "mx_quant", "mx_linear",
                "probe_mfma", "probe_read"]

EXPORTS = [
    "moin_create", "moin_destroy", "moin_strerror", "moin_check", "moin_route", "moin_histogram",
    "moin_lora_linear", "moin_plan_create", "moin_plan_destroy", "moin_plan_build",
    "moin_lora_linear_planned", "moin_timing_enable", "moin_timing_reset", "moin_timing_read",
    "moin_kmeans_update", "moin_retain_clusters", "moin_kmeans_fit",
    "moin_cache_create", "moin_cache_destroy", "moin_cache_add_stack", "moin_cache_admit",
    "moin_cache_table", "moin_cache_stats", "moin_lora_linear_ranked", "moin_plan_build_ranked",
    "moin_mx_quantize", "moin_lora_linear_mx", "moin_lora_linear_mx_planned",
    "moin_probe_out_len", "moin_probe_mfma_bf16", "moin_probe_mfma_mxfp8", "moin_probe_read", "moin_set_adapter_activation",
    "moin_lora_linear_planned_shared", "moin_route_topk", "moin_merge_adapters",
    "moin_reserve_workspace", "moin_workspace_bytes", "moin_plan_reserve", "moin_route_static",
    "moin_cache_set_overlap", "moin_route_plan",
]
ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "silu": 2, "gelu": 3}
CACHE_STATS = ["batches", "seq_hits", "seq_misses", "loads", "evictions", "overflows", "bytes"]

_lib = None


class MoinError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {_strerror(code)} (code {code})")


def load() -> ctypes.CDLL:
    """Opens libmoin.so; a missing library is a hard error (build it with
    ``python -m paper_2410_09687_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2410_09687_amd.build`; "
            "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i32, i64, u32 = c.c_void_p, c.c_int32, c.c_int64, c.c_uint32
    lib.moin_create.argtypes = [c.POINTER(vp), c.c_int]
    lib.moin_destroy.argtypes = [vp]
    lib.moin_destroy.restype = None
    lib.moin_strerror.argtypes = [c.c_int]
    lib.moin_strerror.restype = c.c_char_p
    lib.moin_check.argtypes = [vp, vp]
    lib.moin_route.argtypes = [vp, vp, vp, i64, i32, i32, c.c_int, vp, u32, vp, vp, vp, vp]
    lib.moin_route_static.argtypes = lib.moin_route.argtypes
    lib.moin_histogram.argtypes = [vp, vp, i64, i32, vp, vp]
    lib.moin_lora_linear.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp, i32, i32, i32, i32,
                                     c.c_float, vp, c.c_int, vp]
    lib.moin_lora_linear_ranked.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp, i32, i32, i32, i32, vp,
                                            c.c_float, vp, c.c_int, vp]
    lib.moin_mx_quantize.argtypes = [vp, vp, i64, i64, vp, vp, i32, vp]
    lib.moin_lora_linear_mx.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp, vp, i32, i32, i32, i32, vp,
                                        c.c_float, vp, c.c_int, vp]
    lib.moin_lora_linear_mx_planned.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, i32, i32, i32, c.c_float,
                                                vp, c.c_int, vp]
    lib.moin_set_adapter_activation.argtypes = [vp, i32]
    lib.moin_merge_adapters.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, i32, i32, vp, vp, vp]
    lib.moin_route_topk.argtypes = [vp, vp, vp, i64, i32, i32, c.c_int, vp, c.c_uint32, i32, vp, vp, vp, vp]
    lib.moin_lora_linear_planned_shared.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, vp, i32, c.c_float, vp,
                                                    c.c_int, vp]
    lib.moin_reserve_workspace.argtypes = [vp, i64, vp]
    lib.moin_workspace_bytes.argtypes = [vp]
    lib.moin_plan_reserve.argtypes = [vp, vp, i32, i64, i32, vp]
    lib.moin_probe_out_len.argtypes = [vp]
    lib.moin_probe_out_len.restype = c.c_int64
    lib.moin_probe_mfma_bf16.argtypes = [vp, vp, i64, i32, vp, c.POINTER(c.c_double), vp]
    lib.moin_probe_mfma_mxfp8.argtypes = [vp, vp, i64, i32, vp, c.POINTER(c.c_double), vp]
    lib.moin_probe_read.argtypes = [vp, vp, i64, vp, vp]
    lib.moin_plan_build_ranked.argtypes = [vp, vp, vp, vp, i32, i64, i32, vp, vp]
    lib.moin_route_plan.argtypes = [vp, vp, vp, vp, i64, i32, i32, c.c_int, vp, c.c_uint32, vp, i64, i32, vp,
                                    vp, vp, vp, vp]
    lib.moin_plan_create.argtypes = [vp, c.POINTER(vp)]
    lib.moin_plan_destroy.argtypes = [vp]
    lib.moin_plan_destroy.restype = None
    lib.moin_plan_build.argtypes = [vp, vp, vp, vp, i32, i64, i32, vp]
    lib.moin_lora_linear_planned.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, c.c_float, vp,
                                             c.c_int, vp]
    lib.moin_kmeans_update.argtypes = [vp, vp, vp, i64, vp, i32, i32, c.c_int, vp, c.c_int, vp, vp, vp]
    lib.moin_retain_clusters.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.moin_kmeans_fit.argtypes = [vp, vp, i64, vp, i32, i32, c.c_int, i32, vp, vp, vp, vp]
    lib.moin_cache_create.argtypes = [c.POINTER(vp), i32, i32]
    lib.moin_cache_destroy.argtypes = [vp]
    lib.moin_cache_destroy.restype = None
    lib.moin_cache_add_stack.argtypes = [vp, vp, vp, vp, vp, i64, i64]
    lib.moin_cache_admit.argtypes = [vp, vp, i32, vp, vp]
    lib.moin_cache_set_overlap.argtypes = [vp, c.c_int]
    lib.moin_cache_table.argtypes = [vp, vp, vp]
    lib.moin_cache_stats.argtypes = [vp, vp]
    lib.moin_timing_enable.argtypes = [vp, c.c_int]
    lib.moin_timing_reset.argtypes = [vp]
    lib.moin_timing_read.argtypes = [vp, c.c_int, c.POINTER(c.c_double), c.POINTER(i64)]
    for name in EXPORTS:
        if name not in ("moin_destroy", "moin_plan_destroy", "moin_strerror", "moin_cache_destroy",
                        "moin_probe_out_len", "moin_workspace_bytes"):
            getattr(lib, name).restype = c.c_int
    lib.moin_workspace_bytes.restype = c.c_int64
    _lib = lib
    return lib


def _strerror(code: int) -> str:
    return load().moin_strerror(int(code)).decode()


def _ck(code: int, what: str):
    if code != 0:
        raise MoinError(code, what)


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class Context:
    """Owns a ``moin_ctx`` (workspace, sticky error word, timing slots)."""

    def __init__(self, device: int = 0):
        self._h = ctypes.c_void_p()
        _ck(load().moin_create(ctypes.byref(self._h), int(device)), "moin_create")
        self.device = int(device)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            load().moin_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def check(self, stream=None) -> None:
        """Synchronises the stream; raises ``MoinError`` on a device-side data fault."""
        _ck(load().moin_check(self._h, _stream_ptr(stream)), "moin_check")

    def set_adapter_activation(self, activation=None):
        """Activation between the adapter's two linear layers for every later linear call on this context:
        None (the paper's adapter), "relu", "silu" or "gelu"."""
        if activation not in ACTIVATIONS:
            raise ValueError("activation: None, 'relu', 'silu' or 'gelu' expected")
        _ck(load().moin_set_adapter_activation(self._h, ACTIVATIONS[activation]), "moin_set_adapter_activation")

    def reserve_workspace(self, nbytes: int, stream=None):
        """Grows the workspace to at least ``nbytes`` (outside a stream capture)."""
        _ck(load().moin_reserve_workspace(self._h, int(nbytes), _stream_ptr(stream)), "moin_reserve_workspace")

    def workspace_bytes(self) -> int:
        return int(load().moin_workspace_bytes(self._h))

    def timing_enable(self, on: bool = True):
        _ck(load().moin_timing_enable(self._h, int(on)), "moin_timing_enable")

    def timing_reset(self):
        _ck(load().moin_timing_reset(self._h), "moin_timing_reset")

    def timing_read(self, kernel_id: int):
        ms, n = ctypes.c_double(0), ctypes.c_int64(0)
        _ck(load().moin_timing_read(self._h, int(kernel_id), ctypes.byref(ms), ctypes.byref(n)),
            "moin_timing_read")
        return ms.value, n.value


def moin_route(ctx: Context, emb: torch.Tensor, centroids: torch.Tensor,
               slot_of_centroid: Optional[torch.Tensor] = None, retained_only: bool = False,
               want_centroid_ids: bool = True, want_counts: bool = False, stream=None, out=None,
               static: bool = False, same_centroids: bool = False):
    """Returns ``(expert_ids, centroid_ids or None, counts or None)`` as int32 tensors.  ``out``: the same
    triple preallocated by the caller.  ``static``: through ``moin_route_static``, the entry point that
    allocates no device memory (N <= 65536, K <= 16384).  ``same_centroids``: the caller vouches that
    the table is unchanged since the previous call on this context (``MOIN_ROUTE_SAME_CENTROIDS``)."""
    if emb.dim() != 2 or centroids.dim() != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] expected")
    if emb.dtype != centroids.dtype or emb.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("emb/centroids must both be float32 or both bfloat16")
    N, D = emb.shape
    K = centroids.shape[0]
    dt = MOIN_BF16 if emb.dtype == torch.bfloat16 else MOIN_F32
    dev = centroids.device
    if out is not None:
        expert_ids, cids, counts = out
        for t, n in ((expert_ids, N), (cids, N), (counts, K)):
            if t is not None and (t.dtype != torch.int32 or t.numel() != n):
                raise ValueError("out: int32 tensors of N, N and K elements (or None) expected")
    else:
        expert_ids = torch.empty(N, dtype=torch.int32, device=dev)
        cids = torch.empty(N, dtype=torch.int32, device=dev) if want_centroid_ids else None
        counts = torch.empty(K, dtype=torch.int32, device=dev) if want_counts else None
    fn = load().moin_route_static if static else load().moin_route
    _ck(fn(ctx._h, _dev_ptr(emb, "emb") if N else None, _dev_ptr(centroids, "centroids"),
                          N, K, D, dt, _dev_ptr(slot_of_centroid, "slot_of_centroid", torch.int32),
                          (MOIN_ROUTE_RETAINED_ONLY if retained_only else 0)
                          | (MOIN_ROUTE_SAME_CENTROIDS if same_centroids else 0),
                          _dev_ptr(expert_ids, "expert_ids") if N else None,
                          _dev_ptr(cids, "centroid_ids") if (cids is not None and N) else None,
                          _dev_ptr(counts, "counts"), _stream_ptr(stream)),
        "moin_route_static" if static else "moin_route")
    return expert_ids, cids, counts


def moin_route_topk(ctx: Context, emb: torch.Tensor, centroids: torch.Tensor, k: int,
                    slot_of_centroid: Optional[torch.Tensor] = None, retained_only: bool = False, stream=None):
    """The ``k`` (1..8) nearest centroids of every query, nearest first: ``(expert_ids, centroid_ids, dist2)``,
    each ``[N, k]`` (int32, int32, float32); -1 / inf where fewer than ``k`` centroids took part."""
    if emb.dim() != 2 or centroids.dim() != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] expected")
    if emb.dtype != centroids.dtype or emb.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("emb/centroids must both be float32 or both bfloat16")
    if not 1 <= int(k) <= 8:
        raise ValueError("k must be 1..8")
    N, D = emb.shape
    K = centroids.shape[0]
    dt = MOIN_BF16 if emb.dtype == torch.bfloat16 else MOIN_F32
    dev = centroids.device
    eids = torch.empty((N, k), dtype=torch.int32, device=dev)
    cids = torch.empty((N, k), dtype=torch.int32, device=dev)
    d2 = torch.empty((N, k), dtype=torch.float32, device=dev)
    _ck(load().moin_route_topk(ctx._h, _dev_ptr(emb, "emb") if N else None, _dev_ptr(centroids, "centroids"),
                               N, K, D, dt, _dev_ptr(slot_of_centroid, "slot_of_centroid", torch.int32),
                               MOIN_ROUTE_RETAINED_ONLY if retained_only else 0, int(k),
                               _dev_ptr(eids, "expert_ids") if N else None,
                               _dev_ptr(cids, "centroid_ids") if N else None,
                               _dev_ptr(d2, "dist2") if N else None, _stream_ptr(stream)), "moin_route_topk")
    return eids, cids, d2


def moin_merge_adapters(ctx: Context, A_stack: torch.Tensor, B_stack: torch.Tensor, ids: torch.Tensor,
                        weights: torch.Tensor, A_out: torch.Tensor, B_out: torch.Tensor, stream=None):
    """Writes into ``A_out [r_out, d_in]`` / ``B_out [d_out, r_out]`` (e.g. one slot of wider stacks) the adapter
    of rank ``len(ids) * r`` that stands for ``sum_m weights[m] * B[ids[m]] @ A[ids[m]]``; ``ids`` (int32) and
    ``weights`` (float32) live on the device."""
    E, r, d_in = A_stack.shape
    d_out = B_stack.shape[1]
    if tuple(B_stack.shape) != (E, d_out, r):
        raise ValueError("A_stack [E,r,d_in] / B_stack [E,d_out,r] shape mismatch")
    n = ids.numel()
    if weights.numel() != n:
        raise ValueError("one weight per id expected")
    r_out = A_out.shape[0]
    if tuple(A_out.shape) != (r_out, d_in) or tuple(B_out.shape) != (d_out, r_out):
        raise ValueError("A_out [r_out,d_in] / B_out [d_out,r_out] expected")
    bf = torch.bfloat16
    _ck(load().moin_merge_adapters(ctx._h, _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf), E, r,
                                   d_in, d_out, _dev_ptr(ids, "ids", torch.int32),
                                   _dev_ptr(weights, "weights", torch.float32), n, r_out,
                                   _dev_ptr(A_out, "A_out", bf), _dev_ptr(B_out, "B_out", bf), _stream_ptr(stream)),
        "moin_merge_adapters")


def moin_histogram(ctx: Context, ids: torch.Tensor, K: int, stream=None) -> torch.Tensor:
    counts = torch.empty(K, dtype=torch.int32, device=ids.device)
    _ck(load().moin_histogram(ctx._h, _dev_ptr(ids, "ids", torch.int32) if ids.numel() else None,
                              ids.numel(), K, _dev_ptr(counts, "counts"), _stream_ptr(stream)),
        "moin_histogram")
    return counts


def _y_out(x, d_out, y_dtype, out):
    if y_dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("y dtype must be bfloat16 or float32")
    if out is None:
        out = torch.empty((x.shape[0], d_out), dtype=y_dtype, device=x.device)
    elif out.shape != (x.shape[0], d_out) or out.dtype != y_dtype:
        raise ValueError("out has the wrong shape or dtype")
    return out, (MOIN_BF16 if y_dtype == torch.bfloat16 else MOIN_F32)


def _stack_dims(W, A_stack, B_stack):
    d_out, d_in = W.shape
    if A_stack is None or B_stack is None:
        return d_in, d_out, 0, 0
    E, r = A_stack.shape[0], A_stack.shape[1]
    if tuple(A_stack.shape) != (E, r, d_in) or tuple(B_stack.shape) != (E, d_out, r):
        raise ValueError("A_stack [E,r,d_in] / B_stack [E,d_out,r] shape mismatch")
    return d_in, d_out, E, r


def moin_lora_linear(ctx: Context, x: torch.Tensor, seq_offsets: torch.Tensor,
                     expert_ids: torch.Tensor, W: torch.Tensor, A_stack: Optional[torch.Tensor],
                     B_stack: Optional[torch.Tensor], scale: float, y_dtype=torch.bfloat16,
                     out: Optional[torch.Tensor] = None, stream=None,
                     rank_of_expert: Optional[torch.Tensor] = None) -> torch.Tensor:
    """``rank_of_expert`` (int32 [E] on the device, optional): per-expert adapter rank."""
    if x.dim() != 2 or W.dim() != 2 or x.shape[1] != W.shape[1]:
        raise ValueError("x [T,d_in] and W [d_out,d_in] expected")
    d_in, d_out, E, r = _stack_dims(W, A_stack, B_stack)
    if rank_of_expert is not None and rank_of_expert.numel() != E:
        raise ValueError("rank_of_expert must have E entries")
    S = expert_ids.numel()
    if seq_offsets.numel() != S + 1:
        raise ValueError("seq_offsets must have S+1 entries")
    T = x.shape[0]
    y, ydt = _y_out(x, d_out, y_dtype, out)
    bf = torch.bfloat16
    if rank_of_expert is not None:
        _ck(load().moin_lora_linear_ranked(
            ctx._h, _dev_ptr(x, "x", bf) if T else None, _dev_ptr(seq_offsets, "seq_offsets", torch.int32),
            _dev_ptr(expert_ids, "expert_ids", torch.int32) if S else None, S, T, _dev_ptr(W, "W", bf),
            _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf), E, d_in, d_out, r,
            _dev_ptr(rank_of_expert, "rank_of_expert", torch.int32), float(scale),
            _dev_ptr(y, "y") if T else None, ydt, _stream_ptr(stream)), "moin_lora_linear_ranked")
        return y
    _ck(load().moin_lora_linear(
        ctx._h, _dev_ptr(x, "x", bf) if T else None, _dev_ptr(seq_offsets, "seq_offsets", torch.int32),
        _dev_ptr(expert_ids, "expert_ids", torch.int32) if S else None, S, T, _dev_ptr(W, "W", bf),
        _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf), E, d_in, d_out, r,
        float(scale), _dev_ptr(y, "y") if T else None, ydt, _stream_ptr(stream)), "moin_lora_linear")
    return y


def moin_mx_quantize(ctx: Context, values: torch.Tensor, blocked: bool = False, stream=None):
    """MXFP8 codes ``[rows, cols]`` and scale bytes (both uint8) of a bf16 matrix,
    quantised in blocks of 32 along the last axis.  Scales are ``[rows, cols/32]``,
    or with ``blocked`` (cols a multiple of 128) ``[cols/128, rows, 4]``, the layout
    ``moin_lora_linear_mx`` wants for the weight."""
    if values.dim() != 2 or values.shape[1] % 32 or values.shape[1] == 0:
        raise ValueError("values [rows, cols] with cols a positive multiple of 32 expected")
    rows, cols = values.shape
    if blocked and cols % 128:
        raise ValueError("the blocked scale layout needs cols to be a multiple of 128")
    codes = torch.empty((rows, cols), dtype=torch.uint8, device=values.device)
    scales = torch.empty((cols // 128, rows, 4) if blocked else (rows, cols // 32), dtype=torch.uint8,
                         device=values.device)
    _ck(load().moin_mx_quantize(ctx._h, _dev_ptr(values, "values", torch.bfloat16) if rows else None, rows, cols,
                                _dev_ptr(codes, "codes") if rows else None,
                                _dev_ptr(scales, "scales") if rows else None, 1 if blocked else 0,
                                _stream_ptr(stream)),
        "moin_mx_quantize")
    return codes, scales


def moin_lora_linear_mx(ctx: Context, x: torch.Tensor, seq_offsets: torch.Tensor, expert_ids: torch.Tensor,
                        Wq: torch.Tensor, Ws: torch.Tensor, A_stack: Optional[torch.Tensor],
                        B_stack: Optional[torch.Tensor], scale: float, y_dtype=torch.bfloat16,
                        out: Optional[torch.Tensor] = None, stream=None,
                        rank_of_expert: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Routed LoRA linear on an MXFP8 base (``Wq``, ``Ws`` from ``moin_mx_quantize(..., blocked=True)``)."""
    if x.dim() != 2 or Wq.dim() != 2 or x.shape[1] != Wq.shape[1]:
        raise ValueError("x [T,d_in] and Wq [d_out,d_in] expected")
    if Wq.dtype != torch.uint8 or Ws.dtype != torch.uint8 or Wq.shape[1] % 128 or \
            tuple(Ws.shape) != (Wq.shape[1] // 128, Wq.shape[0], 4):
        raise ValueError("Wq [d_out,d_in] / Ws [d_in/128,d_out,4] (blocked layout) uint8 expected")
    d_in, d_out, E, r = _stack_dims(Wq, A_stack, B_stack)
    if rank_of_expert is not None and rank_of_expert.numel() != E:
        raise ValueError("rank_of_expert must have E entries")
    S = expert_ids.numel()
    if seq_offsets.numel() != S + 1:
        raise ValueError("seq_offsets must have S+1 entries")
    T = x.shape[0]
    y, ydt = _y_out(x, d_out, y_dtype, out)
    bf = torch.bfloat16
    _ck(load().moin_lora_linear_mx(
        ctx._h, _dev_ptr(x, "x", bf) if T else None, _dev_ptr(seq_offsets, "seq_offsets", torch.int32),
        _dev_ptr(expert_ids, "expert_ids", torch.int32) if S else None, S, T, _dev_ptr(Wq, "Wq", torch.uint8),
        _dev_ptr(Ws, "Ws", torch.uint8), _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf),
        E, d_in, d_out, r, _dev_ptr(rank_of_expert, "rank_of_expert", torch.int32), float(scale),
        _dev_ptr(y, "y") if T else None, ydt, _stream_ptr(stream)), "moin_lora_linear_mx")
    return y


class Plan:
    """Grouping of one batch by expert, reusable by every projection of a layer."""

    def __init__(self, ctx: Context):
        self.ctx = ctx
        self._h = ctypes.c_void_p()
        _ck(load().moin_plan_create(ctx._h, ctypes.byref(self._h)), "moin_plan_create")
        self.T = self.S = self.E = 0

    def build(self, seq_offsets: torch.Tensor, expert_ids: torch.Tensor, T: int, E: int, stream=None,
              rank_of_expert: Optional[torch.Tensor] = None):
        S = expert_ids.numel()
        if seq_offsets.numel() != S + 1:
            raise ValueError("seq_offsets must have S+1 entries")
        if rank_of_expert is not None and rank_of_expert.numel() != E:
            raise ValueError("rank_of_expert must have E entries")
        _ck(load().moin_plan_build_ranked(self.ctx._h, self._h, _dev_ptr(seq_offsets, "seq_offsets", torch.int32),
                                          _dev_ptr(expert_ids, "expert_ids", torch.int32) if S else None,
                                          S, T, E, _dev_ptr(rank_of_expert, "rank_of_expert", torch.int32),
                                          _stream_ptr(stream)), "moin_plan_build_ranked")
        self.T, self.S, self.E = T, S, E
        return self

    def reserve(self, S: int, T: int, E: int, stream=None):
        """Sizes the plan's buffer for any batch of at most S sequences, T tokens, E experts."""
        _ck(load().moin_plan_reserve(self.ctx._h, self._h, int(S), int(T), int(E), _stream_ptr(stream)),
            "moin_plan_reserve")
        return self

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            load().moin_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moin_route_plan(ctx: Context, plan: Plan, emb: torch.Tensor, centroids: torch.Tensor,
                    seq_offsets: torch.Tensor, T: int, E: int,
                    slot_of_centroid: Optional[torch.Tensor] = None, retained_only: bool = False,
                    rank_of_expert: Optional[torch.Tensor] = None, want_centroid_ids: bool = False,
                    want_counts: bool = False, same_centroids: bool = False, stream=None, out=None):
    """``moin_route`` and ``Plan.build`` on its ids in one call (one launch for a request-sized batch): the
    ``N`` queries are the batch's sequences.  Returns ``(expert_ids, centroid_ids or None, counts or None)``;
    ``plan`` is rebuilt.  ``out``: the same triple preallocated by the caller (``expert_ids`` required)."""
    if emb.dim() != 2 or centroids.dim() != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] expected")
    if emb.dtype != centroids.dtype or emb.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("emb/centroids must both be float32 or both bfloat16")
    N, D = emb.shape
    K = centroids.shape[0]
    if seq_offsets.numel() != N + 1:
        raise ValueError("seq_offsets must have N+1 entries")
    if rank_of_expert is not None and rank_of_expert.numel() != E:
        raise ValueError("rank_of_expert must have E entries")
    dt = MOIN_BF16 if emb.dtype == torch.bfloat16 else MOIN_F32
    dev = centroids.device
    if out is not None:
        expert_ids, cids, counts = out
        if expert_ids is None:
            raise ValueError("out: expert_ids is required")
        for t, n in ((expert_ids, N), (cids, N), (counts, K)):
            if t is not None and (t.dtype != torch.int32 or t.numel() != n):
                raise ValueError("out: int32 tensors of N, N and K elements (or None) expected")
    else:
        expert_ids = torch.empty(N, dtype=torch.int32, device=dev)
        cids = torch.empty(N, dtype=torch.int32, device=dev) if want_centroid_ids else None
        counts = torch.empty(K, dtype=torch.int32, device=dev) if want_counts else None
    _ck(load().moin_route_plan(ctx._h, plan._h, _dev_ptr(emb, "emb") if N else None,
                               _dev_ptr(centroids, "centroids"), N, K, D, dt,
                               _dev_ptr(slot_of_centroid, "slot_of_centroid", torch.int32),
                               (MOIN_ROUTE_RETAINED_ONLY if retained_only else 0)
                               | (MOIN_ROUTE_SAME_CENTROIDS if same_centroids else 0),
                               _dev_ptr(seq_offsets, "seq_offsets", torch.int32), int(T), int(E),
                               _dev_ptr(rank_of_expert, "rank_of_expert", torch.int32),
                               _dev_ptr(expert_ids, "expert_ids"),
                               _dev_ptr(cids, "centroid_ids") if (cids is not None and N) else None,
                               _dev_ptr(counts, "counts"), _stream_ptr(stream)), "moin_route_plan")
    plan.T, plan.S, plan.E = int(T), N, int(E)
    return expert_ids, cids, counts


def moin_lora_linear_planned(ctx: Context, plan: Plan, x: torch.Tensor, W: torch.Tensor,
                             A_stack: Optional[torch.Tensor], B_stack: Optional[torch.Tensor],
                             scale: float, y_dtype=torch.bfloat16, out: Optional[torch.Tensor] = None,
                             stream=None) -> torch.Tensor:
    if x.dim() != 2 or W.dim() != 2 or x.shape[1] != W.shape[1] or x.shape[0] != plan.T:
        raise ValueError("x [T,d_in] (T as planned) and W [d_out,d_in] expected")
    d_in, d_out, E, r = _stack_dims(W, A_stack, B_stack)
    if E and E != plan.E:
        raise ValueError("stack holds a different number of experts than the plan was built for")
    y, ydt = _y_out(x, d_out, y_dtype, out)
    bf = torch.bfloat16
    T = x.shape[0]
    _ck(load().moin_lora_linear_planned(
        ctx._h, plan._h, _dev_ptr(x, "x", bf) if T else None, _dev_ptr(W, "W", bf),
        _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf), d_in, d_out, r,
        float(scale), _dev_ptr(y, "y") if T else None, ydt, _stream_ptr(stream)),
        "moin_lora_linear_planned")
    return y


def moin_lora_linear_mx_planned(ctx: Context, plan: "Plan", x: torch.Tensor, Wq: torch.Tensor, Ws: torch.Tensor,
                                A_stack: Optional[torch.Tensor], B_stack: Optional[torch.Tensor], scale: float,
                                xq: Optional[torch.Tensor] = None, xs: Optional[torch.Tensor] = None,
                                emit: bool = False, y_dtype=torch.bfloat16, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """``moin_lora_linear_mx`` on a plan; ``xq``, ``xs`` let projections that share their input quantise it
    once: the first call fills them (``emit=True``; uint8 [T, d_in] and [d_in/128, T, 4]), the others read them
    (as they read what ``moin_mx_quantize(x, blocked=True)`` returns)."""
    if x.dim() != 2 or Wq.dim() != 2 or x.shape[1] != Wq.shape[1] or x.shape[0] != plan.T:
        raise ValueError("x [T,d_in] (T as planned) and Wq [d_out,d_in] expected")
    if Wq.dtype != torch.uint8 or Ws.dtype != torch.uint8 or Wq.shape[1] % 128 or \
            tuple(Ws.shape) != (Wq.shape[1] // 128, Wq.shape[0], 4):
        raise ValueError("Wq [d_out,d_in] / Ws [d_in/128,d_out,4] (blocked layout) uint8 expected")
    d_in, d_out, E, r = _stack_dims(Wq, A_stack, B_stack)
    if E and E != plan.E:
        raise ValueError("stack holds a different number of experts than the plan was built for")
    T = x.shape[0]
    if (xq is None) != (xs is None):
        raise ValueError("xq and xs go together")
    if xq is not None and (tuple(xq.shape) != (T, d_in) or tuple(xs.shape) != (d_in // 128, T, 4)):
        raise ValueError("xq [T,d_in] / xs [d_in/128,T,4] (blocked layout) expected")
    if emit and xq is None:
        raise ValueError("emit=True needs xq and xs to write to")
    mode = MOIN_MX_X_INTERNAL if xq is None else (MOIN_MX_X_EMIT if emit else MOIN_MX_X_GIVEN)
    y, ydt = _y_out(x, d_out, y_dtype, out)
    bf = torch.bfloat16
    _ck(load().moin_lora_linear_mx_planned(
        ctx._h, plan._h, _dev_ptr(x, "x", bf) if T else None, _dev_ptr(xq, "xq", torch.uint8),
        _dev_ptr(xs, "xs", torch.uint8), mode, _dev_ptr(Wq, "Wq", torch.uint8), _dev_ptr(Ws, "Ws", torch.uint8),
        _dev_ptr(A_stack, "A_stack", bf), _dev_ptr(B_stack, "B_stack", bf), d_in, d_out, r, float(scale),
        _dev_ptr(y, "y") if T else None, ydt, _stream_ptr(stream)), "moin_lora_linear_mx_planned")
    return y


def moin_lora_linear_planned_shared(ctx: Context, plan: "Plan", x: torch.Tensor, Ws, A_stacks, B_stacks, scale: float,
                                    y_dtype=torch.bfloat16, outs=None, stream=None):
    """``moin_lora_linear_planned`` for up to four projections that read the same ``x`` (q, k, v; gate, up):
    lists of weights ``Ws[i] [d_out_i, d_in]`` and of stacks (or ``None`` for both lists); returns the list
    of outputs.  On the prefill path the adapters' first products come out of one pass over ``x``."""
    n = len(Ws)
    if not 1 <= n <= 4:
        raise ValueError("1 to 4 projections expected")
    if (A_stacks is None) != (B_stacks is None):
        raise ValueError("A_stacks and B_stacks go together")
    if A_stacks is not None and (len(A_stacks) != n or len(B_stacks) != n):
        raise ValueError("one A_stack and one B_stack per weight expected")
    dims = [_stack_dims(Ws[i], None if A_stacks is None else A_stacks[i], None if B_stacks is None else B_stacks[i])
            for i in range(n)]
    d_in, E, r = dims[0][0], dims[0][2], dims[0][3]
    if any(d[0] != d_in or d[2] != E or d[3] != r for d in dims):
        raise ValueError("the projections must agree in d_in, E and r")
    if x.dim() != 2 or x.shape[1] != d_in or x.shape[0] != plan.T:
        raise ValueError("x [T,d_in] (T as planned) expected")
    if E and E != plan.E:
        raise ValueError("stacks hold a different number of experts than the plan was built for")
    T = x.shape[0]
    ys, ydt = [], None
    for i in range(n):
        y, ydt = _y_out(x, dims[i][1], y_dtype, None if outs is None else outs[i])
        ys.append(y)
    bf = torch.bfloat16
    vpa = ctypes.c_void_p * n
    def ptrs(ts, name, dtype=None):
        return vpa(*[(_dev_ptr(t, name, dtype).value if t is not None else None) for t in ts])
    _ck(load().moin_lora_linear_planned_shared(
        ctx._h, plan._h, _dev_ptr(x, "x", bf) if T else None, n, ptrs(Ws, "W", bf),
        ptrs(A_stacks, "A_stack", bf) if A_stacks is not None else None,
        ptrs(B_stacks, "B_stack", bf) if B_stacks is not None else None, d_in,
        (ctypes.c_int32 * n)(*[d[1] for d in dims]), r, float(scale), ptrs(ys, "y") if T else vpa(), ydt,
        _stream_ptr(stream)), "moin_lora_linear_planned_shared")
    return ys


def moin_probe_mfma_bf16(ctx: Context, operands: torch.Tensor, iters: int, stream=None):
    """Measurement aid: a loop of bf16 MFMAs alone on ``operands`` (bf16 values; a wave's lanes take 16-byte
    pieces of it as matrix operands).  Returns (per-thread sums, flops of the launch)."""
    if operands.dtype != torch.bfloat16 or operands.numel() % 8 or operands.numel() < 8:
        raise ValueError("operands: bf16, a multiple of 8 values")
    out = torch.empty(int(load().moin_probe_out_len(ctx._h)), dtype=torch.float32, device=operands.device)
    flops = ctypes.c_double(0.0)
    _ck(load().moin_probe_mfma_bf16(ctx._h, _dev_ptr(operands, "operands", torch.bfloat16), operands.numel() * 2,
                                    int(iters), _dev_ptr(out, "out"), ctypes.byref(flops), _stream_ptr(stream)),
        "moin_probe_mfma_bf16")
    return out, flops.value


def moin_probe_mfma_mxfp8(ctx: Context, codes: torch.Tensor, iters: int, stream=None):
    """Measurement aid: a loop of block-scaled FP8 MFMAs alone on ``codes`` (uint8 E4M3 codes, a multiple of 16
    bytes), all block scales 1.  Returns (per-thread sums, flops of the launch)."""
    if codes.dtype != torch.uint8 or codes.numel() % 16 or codes.numel() < 16:
        raise ValueError("codes: uint8, a multiple of 16 bytes")
    out = torch.empty(int(load().moin_probe_out_len(ctx._h)), dtype=torch.float32, device=codes.device)
    flops = ctypes.c_double(0.0)
    _ck(load().moin_probe_mfma_mxfp8(ctx._h, _dev_ptr(codes, "codes", torch.uint8), codes.numel(), int(iters),
                                     _dev_ptr(out, "out"), ctypes.byref(flops), _stream_ptr(stream)),
        "moin_probe_mfma_mxfp8")
    return out, flops.value


def moin_probe_read(ctx: Context, src: torch.Tensor, stream=None) -> torch.Tensor:
    """Measurement aid: one streaming read of ``src``; returns the per-thread sums (mod 2^32, as int32) of
    the 32-bit words read."""
    nbytes = src.numel() * src.element_size()
    if nbytes % 16 or not src.is_contiguous():
        raise ValueError("src: contiguous, a multiple of 16 bytes")
    out = torch.empty(int(load().moin_probe_out_len(ctx._h)), dtype=torch.int32, device=src.device)
    _ck(load().moin_probe_read(ctx._h, _dev_ptr(src, "src"), nbytes, _dev_ptr(out, "out"), _stream_ptr(stream)),
        "moin_probe_read")
    return out


def _emb_dt(emb, centroids):
    if emb.dim() != 2 or centroids.dim() != 2 or emb.shape[1] != centroids.shape[1]:
        raise ValueError("emb [N,D] and centroids [K,D] expected")
    if emb.dtype != centroids.dtype or emb.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("emb/centroids must both be float32 or both bfloat16")
    return MOIN_BF16 if emb.dtype == torch.bfloat16 else MOIN_F32


def moin_kmeans_update(ctx: Context, emb: torch.Tensor, ids: torch.Tensor, centroids: torch.Tensor,
                       out_dtype=None, out: Optional[torch.Tensor] = None, want_centroids: bool = True,
                       want_counts: bool = True, want_inertia: bool = True, stream=None):
    """Returns ``(new_centroids or None, counts or None, inertia or None)``;
    inertia is a 1-element float64 tensor on the device."""
    dt = _emb_dt(emb, centroids)
    N, D = emb.shape
    K = centroids.shape[0]
    if ids.numel() != N:
        raise ValueError("ids must have N entries")
    dev = centroids.device
    new = None
    odt = dt
    if want_centroids:
        if out is not None:
            new = out
            if new.shape != centroids.shape:
                raise ValueError("out must have the shape of centroids")
        else:
            new = torch.empty((K, D), dtype=out_dtype or centroids.dtype, device=dev)
        if new.dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("new centroids must be float32 or bfloat16")
        odt = MOIN_BF16 if new.dtype == torch.bfloat16 else MOIN_F32
    counts = torch.empty(K, dtype=torch.int32, device=dev) if want_counts else None
    inertia = torch.empty(1, dtype=torch.float64, device=dev) if want_inertia else None
    _ck(load().moin_kmeans_update(
        ctx._h, _dev_ptr(emb, "emb") if N else None, _dev_ptr(ids, "ids", torch.int32) if N else None, N,
        _dev_ptr(centroids, "centroids"), K, D, dt, _dev_ptr(new, "new_centroids"), odt,
        _dev_ptr(counts, "counts"), _dev_ptr(inertia, "inertia"), _stream_ptr(stream)), "moin_kmeans_update")
    return new, counts, inertia


def moin_retain_clusters(ctx: Context, counts: torch.Tensor, min_count: int, stream=None):
    """Returns ``(slot_of_centroid [K] int32, n_retained [1] int32)``."""
    K = counts.numel()
    slot = torch.empty(K, dtype=torch.int32, device=counts.device)
    n = torch.empty(1, dtype=torch.int32, device=counts.device)
    _ck(load().moin_retain_clusters(ctx._h, _dev_ptr(counts, "counts", torch.int32), K, int(min_count),
                                    _dev_ptr(slot, "slot_of_centroid"), _dev_ptr(n, "n_retained"),
                                    _stream_ptr(stream)), "moin_retain_clusters")
    return slot, n


def moin_kmeans_fit(ctx: Context, emb: torch.Tensor, centroids: torch.Tensor, iters: int, stream=None):
    """Runs ``iters`` Lloyd iterations on ``centroids`` IN PLACE; returns
    ``(ids [N], counts [K], inertia [iters + 1] float64)``."""
    dt = _emb_dt(emb, centroids)
    N, D = emb.shape
    K = centroids.shape[0]
    dev = centroids.device
    ids = torch.empty(N, dtype=torch.int32, device=dev)
    counts = torch.empty(K, dtype=torch.int32, device=dev)
    inertia = torch.empty(iters + 1, dtype=torch.float64, device=dev)
    _ck(load().moin_kmeans_fit(ctx._h, _dev_ptr(emb, "emb") if N else None, N, _dev_ptr(centroids, "centroids"),
                               K, D, dt, int(iters), _dev_ptr(ids, "ids") if N else None,
                               _dev_ptr(counts, "counts"), _dev_ptr(inertia, "inertia"), _stream_ptr(stream)),
        "moin_kmeans_fit")
    return ids, counts, inertia


class Cache:
    """Adapter residency cache: ``E`` experts in host memory, ``n_slots`` resident
    on the GPU.  ``add_stack`` registers one projection (host stacks pinned,
    slot stacks on the device); ``admit`` takes a batch's expert ids as a host
    int32 tensor / array and returns the slot ids as a host int32 tensor."""

    def __init__(self, E: int, n_slots: int, overlap: bool = False):
        self._h = ctypes.c_void_p()
        _ck(load().moin_cache_create(ctypes.byref(self._h), int(E), int(n_slots)), "moin_cache_create")
        self.E, self.n_slots = int(E), int(n_slots)
        self._keep = []
        if overlap:
            # copies on the cache's own stream, the previous batch's experts protected: admit batch k+1
            # right after enqueuing the kernels of batch k
            _ck(load().moin_cache_set_overlap(self._h, 1), "moin_cache_set_overlap")

    def add_stack(self, A_host: torch.Tensor, B_host: torch.Tensor, A_slots: torch.Tensor, B_slots: torch.Tensor):
        for t, name in ((A_host, "A_host"), (B_host, "B_host")):
            if t.is_cuda or not t.is_contiguous() or t.shape[0] != self.E:
                raise ValueError(f"{name}: contiguous host tensor with E leading entries expected")
        for t, name in ((A_slots, "A_slots"), (B_slots, "B_slots")):
            if not t.is_cuda or not t.is_contiguous() or t.shape[0] != self.n_slots:
                raise ValueError(f"{name}: contiguous device tensor with n_slots leading entries expected")
        if A_host.shape[1:] != A_slots.shape[1:] or B_host.shape[1:] != B_slots.shape[1:] \
                or A_host.dtype != A_slots.dtype or B_host.dtype != B_slots.dtype:
            raise ValueError("host and slot stacks must agree in per-expert shape and dtype")
        a_bytes = A_host[0].numel() * A_host.element_size()
        b_bytes = B_host[0].numel() * B_host.element_size()
        _ck(load().moin_cache_add_stack(self._h, ctypes.c_void_p(A_host.data_ptr()), ctypes.c_void_p(B_host.data_ptr()),
                                        ctypes.c_void_p(A_slots.data_ptr()), ctypes.c_void_p(B_slots.data_ptr()),
                                        a_bytes, b_bytes), "moin_cache_add_stack")
        self._keep.append((A_host, B_host, A_slots, B_slots))

    def admit(self, expert_ids, stream=None) -> torch.Tensor:
        ids = torch.as_tensor(expert_ids, dtype=torch.int32).contiguous()
        if ids.is_cuda:
            raise ValueError("expert_ids must be a host array (paging is decided on the host)")
        slots = torch.empty_like(ids)
        sp = _stream_ptr(stream) if self._keep else None
        _ck(load().moin_cache_admit(self._h, ctypes.c_void_p(ids.data_ptr()), ids.numel(),
                                    ctypes.c_void_p(slots.data_ptr()), sp), "moin_cache_admit")
        return slots

    def tables(self):
        slot_of = torch.empty(self.E, dtype=torch.int32)
        expert_in = torch.empty(self.n_slots, dtype=torch.int32)
        _ck(load().moin_cache_table(self._h, ctypes.c_void_p(slot_of.data_ptr()),
                                    ctypes.c_void_p(expert_in.data_ptr())), "moin_cache_table")
        return slot_of, expert_in

    def stats(self) -> dict:
        buf = (ctypes.c_int64 * len(CACHE_STATS))()
        _ck(load().moin_cache_stats(self._h, buf), "moin_cache_stats")
        return dict(zip(CACHE_STATS, [int(v) for v in buf]))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            load().moin_cache_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
