"""Helpers shared by the GPU parity tests: move a workload to the GPU, run the
library's pipeline, run the oracle on the same values, compare in original order."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2306_01160_amd import binding as sc
from paper_2306_01160_amd import pipeline, workloads

# tolerances: bf16 inputs with fp32 accumulation (stated by the benchmark definition);
# fp32 path: derived from fp32 rounding of sums over <= 256 keys of O(1) terms
TOL = {"bf16": {"O": 2e-2, "dQ": 2e-2, "dK": 2e-2, "dV": 2e-2, "LSE": 1e-3},
       "f32": {"O": 1e-4, "LSE": 1e-5}}


def to_gpu(wl):
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    q, k, v, do = (torch.from_numpy(a).to(dev).to(tdt) for a in (wl.q, wl.k, wl.v, wl.do))
    lq, lk = (torch.from_numpy(a).to(dev) for a in (wl.lab_q, wl.lab_k))
    return q, k, v, do, lq, lk


def is_strict(wl):
    """workloads tagged meta['strict'] use the strictly-causal mask (keys at earlier positions only)"""
    return bool(wl.meta.get("strict", False))


def run_gpu(wl, backward=True):
    q, k, v, do, lq, lk = to_gpu(wl)
    strict = is_strict(wl)
    if wl.variant == workloads.HASH:
        o, lse, ctx = pipeline.hash_forward(q, k, v, lq, lk, wl.nb, wl.tau, need_bwd=backward, strict=strict)
        grads = pipeline.hash_backward(ctx, do) if backward else None
    else:
        o, lse, ctx = pipeline.qkdrop_forward(q, k, v, lq, lk, wl.tau, need_bwd=backward, strict=strict)
        grads = pipeline.qkdrop_backward(ctx, do) if backward else None
    torch.cuda.synchronize()
    return o, lse, grads, ctx


def seg64(wl, a):
    return a.reshape(wl.S, wl.T, -1).astype(np.float64)


def oracle_variant(wl):
    return oracle.HASH if wl.variant == workloads.HASH else oracle.QKDROP


def labels(wl):
    return wl.lab_q.reshape(wl.S, wl.T).astype(np.int32), wl.lab_k.reshape(wl.S, wl.T).astype(np.int32)


def compare_forward(wl, o, lse, segs=None, rows=None):
    """max-abs errors of O and LSE vs the oracle on the chosen segments / rows."""
    S, T, d = wl.S, wl.T, wl.d
    segs = np.arange(S) if segs is None else np.asarray(segs)
    lq, lk = labels(wl)
    Q, K, V = (seg64(wl, a)[segs] for a in (wl.q, wl.k, wl.v))
    O_ref, L_ref = oracle.attention_forward(Q, K, V, lq[segs], lk[segs], oracle_variant(wl), wl.tau,
                                             strict=is_strict(wl), rows=rows)
    og = o.float().cpu().numpy().reshape(S, T, d)[segs]
    lg = lse.cpu().numpy().reshape(S, T)[segs]
    if rows is not None:
        og, lg = og[:, rows], lg[:, rows]
    fin = np.isfinite(L_ref)
    assert np.array_equal(np.isneginf(lg), ~fin), "rows without keys must have LSE = -inf exactly"
    assert not og[~fin].any(), "rows without keys must be exactly zero"
    err_o = float(np.abs(og - O_ref).max())
    err_l = float(np.abs(lg[fin] - L_ref[fin]).max()) if fin.any() else 0.0
    return {"O": err_o, "LSE": err_l}


def compare_backward(wl, grads, segs=None, q_rows=None, k_rows=None):
    S, T, d = wl.S, wl.T, wl.d
    segs = np.arange(S) if segs is None else np.asarray(segs)
    lq, lk = labels(wl)
    Q, K, V, dO = (seg64(wl, a)[segs] for a in (wl.q, wl.k, wl.v, wl.do))
    dQ_ref, dK_ref, dV_ref = oracle.attention_backward(Q, K, V, dO, lq[segs], lk[segs], oracle_variant(wl),
                                                       wl.tau, strict=is_strict(wl), q_rows=q_rows, k_rows=k_rows)
    out = {}
    for name, g, ref, rows in (("dQ", grads[0], dQ_ref, q_rows), ("dK", grads[1], dK_ref, k_rows),
                               ("dV", grads[2], dV_ref, k_rows)):
        gg = g.cpu().numpy().reshape(S, T, d)[segs]
        if rows is not None:
            gg = gg[:, rows]
        assert np.isfinite(gg).all(), f"{name} has non-finite values"
        out[name] = float(np.abs(gg - ref).max())
    return out


def assert_within(errs, dtype):
    tol = TOL[dtype]
    bad = {k: v for k, v in errs.items() if v > tol[k]}
    assert not bad, f"beyond tolerance: {bad} (all: {errs})"
