"""Shared machinery of the GPU parity tests: run the HIP path through the C-ABI
binding, run the oracle on the same bytes, compare to the stated bars."""
import numpy as np
import torch

import oracle
from paper_2410_09687_amd import moin
from paper_2410_09687_amd import workloads as wl

REL_FRO_MAX = 5e-3     # relative Frobenius error, both output types
MAX_ABS_F32 = 3e-2     # max-abs, fp32 output
# bf16 output: the final rounding alone is half an ulp, which exceeds 3e-2 only
# from |y| = 8 on (2^-5 in [8,16)).  Below 8 the literal 3e-2 holds; from 8 on the
# bar scales with the magnitude.
def bf16_elem_bound(y_ref):
    a = np.abs(y_ref)
    return np.where(a >= 8.0, MAX_ABS_F32 * a / 4.0, MAX_ABS_F32)


_ctx = None


def ctx():
    global _ctx
    if _ctx is None:
        import atexit
        _ctx = moin.Context(0)
        atexit.register(_ctx.close)   # release before the HIP runtime shuts down
    return _ctx


def oracle_rows(inp: wl.LinearInputs, rows=None, expert_ids=None):
    """Oracle output for the chosen token rows (all when None), fed with host
    copies of exactly the bytes the GPU consumed."""
    A, B, ids = wl.compact_stacks(inp) if expert_ids is None else expert_ids
    return oracle.lora_linear(wl.bf16_bits(inp.x), inp.seq_offsets.cpu().numpy(), ids,
                              wl.bf16_bits(inp.W), A, B, inp.wl.scale, rows=rows)


def compare_linear(y_gpu: torch.Tensor, y_ref: np.ndarray, rows=None, what=""):
    y = y_gpu.detach().float().cpu().double().numpy()
    if rows is not None:
        y = y[np.asarray(rows)]
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    if y_ref.size == 0:
        return {}
    assert np.isfinite(y).all(), f"{what}: non-finite output"
    err = np.abs(y - y_ref)
    fro = np.linalg.norm(y - y_ref) / max(np.linalg.norm(y_ref), 1e-30)
    stats = {"rel_fro": float(fro), "max_abs": float(err.max())}
    assert fro <= REL_FRO_MAX, f"{what}: rel Frobenius {fro:.3e} > {REL_FRO_MAX}"
    if y_gpu.dtype == torch.float32:
        assert err.max() <= MAX_ABS_F32, f"{what}: max-abs {err.max():.3e} > {MAX_ABS_F32}"
    else:
        over = err > bf16_elem_bound(y_ref)
        assert not over.any(), f"{what}: {int(over.sum())} elements beyond the bf16 bound, worst {err.max():.3e}"
    return stats


def run_linear(inp: wl.LinearInputs, y_dtype=torch.bfloat16):
    y = moin.moin_lora_linear(ctx(), inp.x, inp.seq_offsets, inp.expert_ids, inp.W, inp.A_stack,
                                 inp.B_stack, inp.wl.scale, y_dtype=y_dtype)
    ctx().check()
    return y


def check_route(emb: torch.Tensor, cent: torch.Tensor, ids_gpu: torch.Tensor, sample=None,
                eligible=None):
    """Exact ids, except where the GPU's pick lies within 1e-4 (relative, on the
    squared distance, fp64) of the true minimum.  Returns the number accepted
    inside that band."""
    to_host = (lambda t: wl.bf16_bits(t)) if emb.dtype == torch.bfloat16 else (lambda t: t.cpu().numpy())
    sel = np.arange(emb.shape[0]) if sample is None else np.asarray(sample)
    q = to_host(emb[torch.as_tensor(sel, device=emb.device)]) if sample is not None else to_host(emb)
    c = to_host(cent)
    ref, best, _ = oracle.route(q, c, eligible=eligible, want_gaps=True)
    got = ids_gpu.cpu().numpy()[sel]
    assert got.min(initial=0) >= 0 and got.max(initial=0) < c.shape[0]
    bad = np.flatnonzero(got != ref)
    if bad.size:
        if eligible is not None:
            assert np.asarray(eligible)[got[bad]].all(), "routed to a centroid outside the search"
        d = oracle.dist2(q, c, bad, got[bad])
        lim = np.where(best[bad] > 0, best[bad] * (1 + 1e-4), 1e-30)
        worst = bad[d > lim]
        assert worst.size == 0, f"{worst.size} ids differ outside the near-tie band (first: query {sel[worst[0]]})"
    return int(bad.size)
