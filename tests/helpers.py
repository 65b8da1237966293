"""Shared pieces of the GPU parity tests: run a block on the GPU through the C ABI,
run the same block on the oracle, compare tensor by tensor."""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

import d2ft_inputs as di

GRAD_FIELDS_ALL = di.WEIGHT_FIELDS

# Tolerances of the parity bar: max |gpu - oracle| / max |oracle| per tensor.
TOL = {"f32": 1e-4, "bf16": 2e-2}


def rel_inf(got: np.ndarray, ref: np.ndarray) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


FLAG_GATE_FFN = 4   # the op code of a head also governs its 1/H slice of the feed-forward network


def oracle_block(w: di.Workload, weights: Dict[str, Optional[np.ndarray]], ops: Sequence[int], x, dy,
                 gate_ffn: bool = False):
    from oracle import d2ft_oracle as orc
    y, cache = orc.block_fwd(weights, ops, x, w.head_dim, w.ln_eps, w.lora_scale, gate_ffn=gate_ffn)
    dx, g = orc.block_bwd(weights, cache, dy)
    return y, dx, g, cache


def gpu_block(w: di.Workload, weights: Dict[str, Optional[np.ndarray]], ops: Sequence[int], x, dy,
              grad_fields=GRAD_FIELDS_ALL, flags: int = 0, grads_init: Optional[Dict[str, np.ndarray]] = None):
    """One block forward + backward through libd2ft.  Returns host fp32 arrays (y, dx, grads)."""
    import torch
    import paper_2504_12471_amd as P
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, flags)
    dw = {k: P.to_device(v, w.dtype) for k, v in weights.items()}
    tdt = P.torch_dtype(w.dtype)
    xd, dyd = P.to_device(x, w.dtype), P.to_device(dy, w.dtype)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    saved = torch.empty(P.d2ft_block_saved_bytes(desc), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(P.d2ft_block_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    grads = {}
    for k in di.WEIGHT_FIELDS:
        if k in grad_fields and dw.get(k) is not None:
            if grads_init is not None and k in grads_init:
                grads[k] = P.to_device(grads_init[k], w.dtype)
            else:
                # poison: overwrite mode must replace every element
                grads[k] = torch.full_like(dw[k], float("nan"))
        else:
            grads[k] = None
    P.d2ft_block_fwd(desc, dw, ops, xd, y, saved, scratch)
    P.d2ft_block_bwd(desc, dw, ops, xd, dyd, dx, grads, saved, scratch)
    torch.cuda.synchronize()
    host = lambda t: None if t is None else t.float().cpu().numpy()
    return host(y), host(dx), {k: host(v) for k, v in grads.items()}


def compare_block(w: di.Workload, ops, got, ref, tol: float, grad_fields=GRAD_FIELDS_ALL, report=None,
                  gate_ffn: bool = False):
    """got = (y, dx, grads) from the GPU, ref = (y, dx, grads) from the oracle."""
    y, dx, g = got
    ry, rdx, rg = ref[:3]
    errs = {"y": rel_inf(y, ry), "dx": rel_inf(dx, rdx)}
    dh = w.head_dim
    for k in grad_fields:
        if g.get(k) is None:
            continue
        assert np.all(np.isfinite(g[k])), f"{k}: non-finite (an element was not written)"
        errs["d" + k] = rel_inf(g[k], rg[k])
    if report is not None:
        report.update(errs)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"over tolerance {tol}: {bad}  (all: {errs})"
    # heads that are not p_f: every gradient slice is exactly +0.0
    for h, o in enumerate(ops):
        if o == di.OP_FULL:
            continue
        slices = []
        if g.get("w_qkv") is not None: slices.append(g["w_qkv"][:, h])
        if g.get("b_qkv") is not None: slices.append(g["b_qkv"][:, h])
        if g.get("w_o") is not None: slices.append(g["w_o"][:, h * dh:(h + 1) * dh])
        for k in ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"):
            if g.get(k) is not None: slices.append(g[k][h])
        if gate_ffn:
            S = w.mlp_hidden // w.heads
            if g.get("w1") is not None: slices.append(g["w1"][h * S:(h + 1) * S])
            if g.get("b1") is not None: slices.append(g["b1"][h * S:(h + 1) * S])
            if g.get("w2") is not None: slices.append(g["w2"][:, h * S:(h + 1) * S])
        for s in slices:
            assert np.all(s == 0.0) and not np.any(np.signbit(s)), f"head {h} (op {o}) has a non-zero gradient"
    return errs
