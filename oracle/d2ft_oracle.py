"""CPU fp64 oracle for the head-selective ViT block and the bi-level knapsack.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
GPU library is checked against.  It shares no code with the HIP path, and only
the tests, the smoke check and the benchmark's cpu_baseline leg may import it.

What it follows:
  * Operation set P = {p_f full, p_o forward-only, p_s shortcut} and the
    residual route (Sec. II-A.2 "Operation selection").
  * Partition of a block into per-head subnets (Sec. II-A.1).
  * KnapsackScheduling and DPSearching (Alg. 1 and Alg. 2, Sec. II-C), the
    bi-level problem they solve (Eq. 4 and Eq. 5).
  * The LoRA extension: per-head adapters, base frozen (Sec. II-D).
  * The analytic cost rules (Sec. IV-A "Analysis of computational and
    communicational cost").
  * The two contribution scores of a subnet (Sec. II-B "Contribution scores"):
    Fisher information (sum of squared gradient entries) and weight magnitude.

Readings taken where the paper is silent or garbled (each also listed in the
design notes of the repository):
  * p_o is a stop-gradient on the head's output: no weight gradient and no
    input gradient flows through a forward-only head (it costs only a forward
    pass and sends no backward message, Sec. IV-A).
  * p_s removes the head's term from the concatenation, i.e. its Q/K/V
    columns and its output-projection columns are dropped.
  * The output-projection bias is added iff at least one head is live, so an
    all-shortcut block leaves the attention residual untouched.
  * LayerNorm uses the biased variance; GELU is the exact erf form.
  * By default the feed-forward network is not gated: it always runs forward
    and backward.  With gate_ffn the subnet of Sec. II-A.1 is taken whole: head
    h owns hidden units [h*Dm/H, (h+1)*Dm/H) of the feed-forward network (the
    1/H part the paper assigns to it, Sec. IV-A "Full fine-tuning partition
    settings") and the head's op code applies to that slice too: p_s drops the
    slice, p_o keeps its forward term as a constant, p_f trains it.  The second
    layer's bias is added iff at least one slice is live, the same rule as for
    the output-projection bias, so an all-shortcut block is the identity.
  * "Weight magnitude" is the sum of absolute values of the subnet's weights.
    A subnet's tensors are the slices that belong to one head alone: its
    Q/K/V weight rows and biases, its output-projection columns, its LoRA
    adapters, and (whole-subnet gating) its feed-forward slice.  LayerNorm
    parameters (frozen and replicated, Sec. IV-A) and the two shared output
    biases belong to no single subnet and are left out.
  * Micro-batches: the scheduling table holds one code per (subnet, micro-batch)
    (Alg. 1, T_opt[k][x_i]); a block call over several micro-batches applies
    each micro-batch's codes to its own images, and a weight gradient is the
    sum of the micro-batches' gradients (gradient accumulation).
  * The optimizer is SGD with momentum (Sec. IV-A names it and gives no
    hyper-parameters): v <- mu*v + (g + wd*w), w <- w - lr*v, the common
    formulation without dampening or Nesterov look-ahead.  Slices that belong to
    a subnet that was not p_f in the step are left untouched, momentum included
    (a device that skipped its subnet does no work on it); tensors shared by all
    subnets are always updated.
  * The two subnets outside the blocks (Sec. IV-A "Full fine-tuning partition
    settings": the patch embedding layer, and the global pooling and
    classification layer) are taken in the usual ViT form, which the paper does
    not spell out: non-overlapping P x P patches flattened in (channel, row,
    column) order and projected linearly, a class token in front, learned
    position embeddings added; at the end LayerNorm of the class token (the
    pooling), a linear layer and mean softmax cross-entropy.
  * In DPSearching the item weight tested and subtracted in the fill phase is
    the operation's own weight (W_p), as the backtracking phase uses; the
    backtracking index decrements by one.
  * An item is taken only where it strictly changes the table value.  What the
    selection does on exactly tied scores rests on that rule alone: parity
    unpinned for ties (every other part of this file has a pin in tests/).
  * The two DP calls use separate capacities, as Alg. 1's inputs state; an
    item chosen by both is p_f.

All arithmetic is float64.  Every function is written as the definition, with
loops over heads; there is no blocking, fusion or reordering.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

OP_FULL, OP_FWD, OP_SKIP = 1, 2, 3   # codes of the scheduling table, Alg. 1


# ----------------------------------------------------------------------------
# head compaction
# ----------------------------------------------------------------------------
def compact_heads(ops: Sequence[int]) -> Tuple[List[int], int, int]:
    """Live-head list of one block: full heads ascending, then forward-only heads ascending.

    Returns (live, n_full, n_live).  Shortcut heads do not appear.
    (Sec. II-A.2: p_f and p_o run the forward pass, p_s bypasses the subnet.)
    """
    full, fwd = [], []
    for h, code in enumerate(ops):
        code = int(code)
        if code == OP_FULL:
            full.append(h)
        elif code == OP_FWD:
            fwd.append(h)
        elif code != OP_SKIP:
            raise ValueError(f"bad op code {code} at head {h}")
    return full + fwd, len(full), len(full) + len(fwd)


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------
def layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float):
    """Per-row LayerNorm with biased variance.  Returns (y, xhat, rstd)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, xhat, rstd


def layer_norm_bwd(d: np.ndarray, xhat: np.ndarray, rstd: np.ndarray, gamma: np.ndarray):
    """Gradient of layer_norm.  Returns (dx, dgamma, dbeta)."""
    dhat = d * gamma
    m1 = dhat.mean(axis=-1, keepdims=True)
    m2 = (dhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dhat - m1 - xhat * m2)
    D = d.shape[-1]
    return dx, (d * xhat).reshape(-1, D).sum(axis=0), d.reshape(-1, D).sum(axis=0)


def gelu(z: np.ndarray) -> np.ndarray:
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def gelu_grad(z: np.ndarray) -> np.ndarray:
    cdf = 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    return cdf + z * pdf


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------
# block forward
# ----------------------------------------------------------------------------
def block_fwd(w: Dict[str, Optional[np.ndarray]], ops: Sequence[int], x: np.ndarray,
              head_dim: int, ln_eps: float = 1e-6, lora_scale: float = 1.0,
              attn_const: Optional[np.ndarray] = None, gate_ffn: bool = False,
              ffn_const: Optional[np.ndarray] = None):
    """Forward of one pre-LN block whose heads carry op codes.

    x: [B, T, D].  w: arrays named as in the library's weight struct
    (w_qkv [3,H,dh,D], b_qkv [3,H,dh], w_o [D,H*dh], b_o [D] or None, w1 [Dm,D],
    w2 [D,Dm], optional lora_a_q/v [H,r,D], lora_b_q/v [H,dh,r]).
    attn_const, if given, is a [B, T, D] constant added to the attention
    residual; a test uses it to hold a forward-only head's output fixed while
    it perturbs parameters (the stop-gradient reading of p_o); ffn_const does
    the same for the feed-forward residual.
    gate_ffn: head h's op code also governs hidden units [h*Dm/H, (h+1)*Dm/H)
    of the feed-forward network (the subnet of Sec. II-A.1).
    Returns (y, cache); cache holds what block_bwd needs.
    """
    w = {k: _f64(v) for k, v in w.items()}
    x = _f64(x)
    B, T, D = x.shape
    dh = head_dim
    live, n_full, n_live = compact_heads(ops)
    has_lora = w.get("lora_a_q") is not None
    cache = {"x": x, "ops": list(int(o) for o in ops), "live": live, "n_full": n_full,
             "heads": {}}

    attn = np.zeros_like(x)
    if n_live > 0:
        u, xhat1, rstd1 = layer_norm(x, w["ln1_g"], w["ln1_b"], ln_eps)
        cache.update(u=u, xhat1=xhat1, rstd1=rstd1)
        for h in live:
            q = u @ w["w_qkv"][0, h].T + w["b_qkv"][0, h]
            k = u @ w["w_qkv"][1, h].T + w["b_qkv"][1, h]
            v = u @ w["w_qkv"][2, h].T + w["b_qkv"][2, h]
            if has_lora:
                q = q + lora_scale * ((u @ w["lora_a_q"][h].T) @ w["lora_b_q"][h].T)
                v = v + lora_scale * ((u @ w["lora_a_v"][h].T) @ w["lora_b_v"][h].T)
            s = (q @ np.swapaxes(k, -1, -2)) / math.sqrt(dh)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            p = e / e.sum(axis=-1, keepdims=True)
            o = p @ v
            contrib = o @ w["w_o"][:, h * dh:(h + 1) * dh].T
            attn = attn + contrib
            cache["heads"][h] = dict(q=q, k=k, v=v, p=p, o=o, contrib=contrib)
        if w.get("b_o") is not None:
            attn = attn + w["b_o"]
        x1 = x + attn
    else:
        x1 = x.copy()
    if attn_const is not None:
        x1 = x1 + _f64(attn_const)

    cache.update(x1=x1, head_dim=dh, lora_scale=lora_scale, has_lora=has_lora, gate_ffn=gate_ffn)
    if not gate_ffn:
        vv, xhat2, rstd2 = layer_norm(x1, w["ln2_g"], w["ln2_b"], ln_eps)
        z = vv @ w["w1"].T + w["b1"]
        g = gelu(z)
        y = x1 + g @ w["w2"].T
        if w.get("b2") is not None:
            y = y + w["b2"]
        cache.update(v=vv, xhat2=xhat2, rstd2=rstd2, z=z, g=g)
    else:
        Dm = w["w1"].shape[0]
        if Dm % len(ops) != 0:
            raise ValueError("the hidden width must divide evenly over the heads")
        S = Dm // len(ops)
        ffn = np.zeros_like(x1)
        cache["slices"] = {}
        if n_live > 0:
            vv, xhat2, rstd2 = layer_norm(x1, w["ln2_g"], w["ln2_b"], ln_eps)
            cache.update(v=vv, xhat2=xhat2, rstd2=rstd2)
            for h in live:
                sl = slice(h * S, (h + 1) * S)
                z = vv @ w["w1"][sl].T + w["b1"][sl]
                g = gelu(z)
                ffn = ffn + g @ w["w2"][:, sl].T
                cache["slices"][h] = dict(z=z, g=g)
            if w.get("b2") is not None:
                ffn = ffn + w["b2"]
        y = x1 + ffn
    if ffn_const is not None:
        y = y + _f64(ffn_const)
    return y, cache


# ----------------------------------------------------------------------------
# block backward
# ----------------------------------------------------------------------------
def block_bwd(w: Dict[str, Optional[np.ndarray]], cache: dict, dy: np.ndarray):
    """Backward of block_fwd given dy.  Returns (dx, grads).

    grads has one array per weight field, the same shape as the weight.  Slices
    that belong to forward-only or shortcut heads are exactly zero: p_o keeps
    the forward pass but skips backward propagation, p_s skips both
    (Sec. II-A.2), and the gradient reaches earlier blocks by the residual
    route alone.
    """
    w = {k: _f64(v) for k, v in w.items()}
    dy = _f64(dy)
    x = cache["x"]
    B, T, D = x.shape
    dh = cache["head_dim"]
    s_l = cache["lora_scale"]
    live, n_full = cache["live"], cache["n_full"]
    full = live[:n_full]
    rows = lambda a: a.reshape(-1, a.shape[-1])

    g = {k: (None if v is None else np.zeros_like(v)) for k, v in w.items()}

    if not cache["gate_ffn"]:
        # feed-forward network, not gated
        g["w2"] = rows(dy).T @ rows(cache["g"])
        if w.get("b2") is not None:
            g["b2"] = rows(dy).sum(axis=0)
        dg = dy @ w["w2"]
        dz = dg * gelu_grad(cache["z"])
        g["w1"] = rows(dz).T @ rows(cache["v"])
        g["b1"] = rows(dz).sum(axis=0)
        dv = dz @ w["w1"]
        dln2, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dv, cache["xhat2"], cache["rstd2"], w["ln2_g"])
        dx1 = dy + dln2
    else:
        # feed-forward slices of the p_f subnets only; the others leave exact zeros (Sec. II-A.2)
        S = w["w1"].shape[0] // len(cache["ops"])
        if len(live) > 0 and w.get("b2") is not None:
            g["b2"] = rows(dy).sum(axis=0)
        if n_full == 0:
            dx1 = dy.copy()
        else:
            dv = np.zeros_like(cache["v"])
            for h in full:
                sl = slice(h * S, (h + 1) * S)
                c = cache["slices"][h]
                g["w2"][:, sl] = rows(dy).T @ rows(c["g"])
                dz = (dy @ w["w2"][:, sl]) * gelu_grad(c["z"])
                g["w1"][sl] = rows(dz).T @ rows(cache["v"])
                g["b1"][sl] = rows(dz).sum(axis=0)
                dv = dv + dz @ w["w1"][sl]
            dln2, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dv, cache["xhat2"], cache["rstd2"], w["ln2_g"])
            dx1 = dy + dln2

    # attention side
    if len(live) > 0 and w.get("b_o") is not None:
        g["b_o"] = rows(dx1).sum(axis=0)
    if n_full == 0:
        return dx1, g

    u = cache["u"]
    du = np.zeros_like(u)
    for h in full:
        c = cache["heads"][h]
        q, k, v, p, o = c["q"], c["k"], c["v"], c["p"], c["o"]
        wo_h = w["w_o"][:, h * dh:(h + 1) * dh]            # [D, dh]
        do = dx1 @ wo_h                                    # [B,T,dh]
        g["w_o"][:, h * dh:(h + 1) * dh] = rows(dx1).T @ rows(o)
        dvh = np.swapaxes(p, -1, -2) @ do
        dp = do @ np.swapaxes(v, -1, -2)
        ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
        dq = (ds @ k) / math.sqrt(dh)
        dk = (np.swapaxes(ds, -1, -2) @ q) / math.sqrt(dh)
        for which, dproj in ((0, dq), (1, dk), (2, dvh)):
            g["w_qkv"][which, h] = rows(dproj).T @ rows(u)
            g["b_qkv"][which, h] = rows(dproj).sum(axis=0)
            du = du + dproj @ w["w_qkv"][which, h]
        if cache["has_lora"]:
            for name, dproj in (("q", dq), ("v", dvh)):
                a, b = w[f"lora_a_{name}"][h], w[f"lora_b_{name}"][h]   # [r,D], [dh,r]
                t = u @ a.T                                              # [B,T,r]
                g[f"lora_b_{name}"][h] = s_l * (rows(dproj).T @ rows(t))
                dt = s_l * (dproj @ b)                                   # [B,T,r]
                g[f"lora_a_{name}"][h] = rows(dt).T @ rows(u)
                du = du + dt @ a
    dln1, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(du, cache["xhat1"], cache["rstd1"], w["ln1_g"])
    return dx1 + dln1, g


# ----------------------------------------------------------------------------
# one block over several micro-batches, each with its own op codes (Alg. 1, T_opt[k][x_i])
# ----------------------------------------------------------------------------
def block_fwd_mb(w, ops_mb: Sequence[Sequence[int]], mb_images: Sequence[int], x: np.ndarray, head_dim: int,
                 ln_eps: float = 1e-6, lora_scale: float = 1.0, gate_ffn: bool = False):
    """x: [B, T, D] with B = sum(mb_images); micro-batch i is the next mb_images[i] images and runs
    under ops_mb[i].  Returns (y, caches)."""
    x = _f64(x)
    if sum(mb_images) != x.shape[0] or len(ops_mb) != len(mb_images):
        raise ValueError("micro-batch sizes must add up to the batch")
    ys, caches, b0 = [], [], 0
    for ops, nb in zip(ops_mb, mb_images):
        y, c = block_fwd(w, ops, x[b0:b0 + nb], head_dim, ln_eps, lora_scale, gate_ffn=gate_ffn)
        ys.append(y)
        caches.append(c)
        b0 += nb
    return np.concatenate(ys, axis=0), caches


def block_bwd_mb(w, caches: List[dict], mb_images: Sequence[int], dy: np.ndarray):
    """Backward of block_fwd_mb: dx per micro-batch, weight gradients summed over the micro-batches."""
    dy = _f64(dy)
    dxs, total, b0 = [], None, 0
    for c, nb in zip(caches, mb_images):
        dx, g = block_bwd(w, c, dy[b0:b0 + nb])
        dxs.append(dx)
        if total is None:
            total = g
        else:
            total = {k: (None if v is None else v + g[k]) for k, v in total.items()}
        b0 += nb
    return np.concatenate(dxs, axis=0), total


# ----------------------------------------------------------------------------
# stack of blocks
# ----------------------------------------------------------------------------
def stack_fwd(weights: List[dict], ops: np.ndarray, x: np.ndarray, head_dim: int,
              ln_eps: float = 1e-6, lora_scale: float = 1.0, gate_ffn: bool = False):
    caches, h = [], _f64(x)
    for l, w in enumerate(weights):
        h, c = block_fwd(w, ops[l], h, head_dim, ln_eps, lora_scale, gate_ffn=gate_ffn)
        caches.append(c)
    return h, caches


def stack_bwd(weights: List[dict], caches: List[dict], dy: np.ndarray):
    grads, d = [None] * len(weights), _f64(dy)
    for l in range(len(weights) - 1, -1, -1):
        d, grads[l] = block_bwd(weights[l], caches[l], d)
    return d, grads


# ----------------------------------------------------------------------------
# contribution scores (Sec. II-B)
# ----------------------------------------------------------------------------
def subnet_scores(t: Dict[str, Optional[np.ndarray]], heads: int, head_dim: int, kind: str,
                  gate_ffn: bool = False) -> np.ndarray:
    """Score of every subnet of one block from tensors in the weight layout.

    kind "fisher": sum of squared entries (t holds the gradients of one sample or
    micro-batch: empirical Fisher information); kind "magnitude": sum of absolute
    values (t holds the weights).  Fields that are None are skipped.
    Returns [heads] float64.
    """
    if kind not in ("fisher", "magnitude"):
        raise ValueError(kind)
    f = (lambda a: float((a * a).sum())) if kind == "fisher" else (lambda a: float(np.abs(a).sum()))
    t = {k: _f64(v) for k, v in t.items()}
    dh = head_dim
    out = np.zeros(heads, dtype=np.float64)
    for h in range(heads):
        parts = []
        if t.get("w_qkv") is not None:
            parts.append(t["w_qkv"][:, h])
        if t.get("b_qkv") is not None:
            parts.append(t["b_qkv"][:, h])
        if t.get("w_o") is not None:
            parts.append(t["w_o"][:, h * dh:(h + 1) * dh])
        for k in ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"):
            if t.get(k) is not None:
                parts.append(t[k][h])
        if gate_ffn:
            S = (t["w1"] if t.get("w1") is not None else t["w2"].T).shape[0] // heads
            if t.get("w1") is not None:
                parts.append(t["w1"][h * S:(h + 1) * S])
            if t.get("b1") is not None:
                parts.append(t["b1"][h * S:(h + 1) * S])
            if t.get("w2") is not None:
                parts.append(t["w2"][:, h * S:(h + 1) * S])
        out[h] = sum(f(a) for a in parts)
    return out


# ----------------------------------------------------------------------------
# SGD with momentum on the slices of the p_f subnets (Sec. IV-A: "SGD optimizer with momentum")
# ----------------------------------------------------------------------------
def _head_slices(name: str, a: np.ndarray, h: int, heads: int, head_dim: int, gate_ffn: bool):
    """Index expression of head h's slice of tensor `name`, or None if the tensor is shared by all heads."""
    if name in ("w_qkv", "b_qkv"):
        return (slice(None), h)
    if name == "w_o":
        return (slice(None), slice(h * head_dim, (h + 1) * head_dim))
    if name.startswith("lora_"):
        return (h,)
    if gate_ffn and name in ("w1", "b1"):
        S = a.shape[0] // heads
        return (slice(h * S, (h + 1) * S),)
    if gate_ffn and name == "w2":
        S = a.shape[1] // heads
        return (slice(None), slice(h * S, (h + 1) * S))
    return None


def sgd_momentum_step(w: Dict[str, Optional[np.ndarray]], g: Dict[str, Optional[np.ndarray]],
                      v: Dict[str, Optional[np.ndarray]], updated: Sequence[bool], head_dim: int,
                      lr: float, momentum: float, weight_decay: float = 0.0, gate_ffn: bool = False):
    """One optimizer step.  w, g, v: weights, gradients, momentum buffers in the weight layout
    (fields that are None in g are not trained).  updated[h]: subnet h was p_f in this step.
    Returns (w_new, v_new) as new float64 dicts; slices of subnets with updated[h] False are copied."""
    heads = len(updated)
    w_new = {k: (None if a is None else np.array(a, dtype=np.float64)) for k, a in w.items()}
    v_new = {k: (None if a is None else np.array(a, dtype=np.float64)) for k, a in v.items()}
    for k, grad in g.items():
        if grad is None or w.get(k) is None:
            continue
        grad = _f64(grad)
        regions = []
        if _head_slices(k, grad, 0, heads, head_dim, gate_ffn) is None:
            regions.append((slice(None),))
        else:
            regions = [_head_slices(k, grad, h, heads, head_dim, gate_ffn) for h in range(heads) if updated[h]]
        for r in regions:
            vv = momentum * v_new[k][r] + (grad[r] + weight_decay * w_new[k][r])
            v_new[k][r] = vv
            w_new[k][r] = w_new[k][r] - lr * vv
    return w_new, v_new


# ----------------------------------------------------------------------------
# the two subnets outside the blocks (Sec. IV-A): patch embedding, pooling + classifier
# ----------------------------------------------------------------------------
def patch_embed_fwd(images: np.ndarray, w_pe: np.ndarray, b_pe: np.ndarray, cls: np.ndarray, pos: np.ndarray,
                    patch: int):
    """images [B, C, H, W] -> tokens [B, 1 + (H/P)(W/P), D].  w_pe [D, C*P*P] with k = (c*P + i)*P + j."""
    images, w_pe, b_pe, cls, pos = map(_f64, (images, w_pe, b_pe, cls, pos))
    B, C, H, W = images.shape
    P = patch
    ny, nx = H // P, W // P
    patches = np.zeros((B, ny * nx, C * P * P))
    for py in range(ny):
        for px in range(nx):
            blk = images[:, :, py * P:(py + 1) * P, px * P:(px + 1) * P]       # [B, C, P, P]
            patches[:, py * nx + px] = blk.reshape(B, -1)
    tokens = np.zeros((B, 1 + ny * nx, w_pe.shape[0]))
    tokens[:, 0] = cls + pos[0]
    tokens[:, 1:] = patches @ w_pe.T + b_pe + pos[1:]
    return tokens, dict(patches=patches)


def patch_embed_bwd(cache: dict, dtokens: np.ndarray):
    """Gradients of the embedding's parameters (no gradient is taken with respect to the images)."""
    dtokens = _f64(dtokens)
    dp = dtokens[:, 1:]
    D = dtokens.shape[-1]
    return dict(w_pe=dp.reshape(-1, D).T @ cache["patches"].reshape(-1, cache["patches"].shape[-1]),
                b_pe=dp.reshape(-1, D).sum(axis=0), cls=dtokens[:, 0].sum(axis=0), pos=dtokens.sum(axis=0))


def classifier_fwd(tokens: np.ndarray, ln_g, ln_b, w_c, b_c, labels: Sequence[int], ln_eps: float = 1e-6):
    """Class-token pooling, LayerNorm, linear layer, mean softmax cross-entropy.  Returns (loss, logits, cache)."""
    tokens, ln_g, ln_b, w_c, b_c = map(_f64, (tokens, ln_g, ln_b, w_c, b_c))
    h, xhat, rstd = layer_norm(tokens[:, 0], ln_g, ln_b, ln_eps)
    logits = h @ w_c.T + b_c
    zmax = logits.max(axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(logits - zmax).sum(axis=-1))
    labels = np.asarray(labels, dtype=np.int64)
    loss = float((lse - logits[np.arange(len(labels)), labels]).mean())
    return loss, logits, dict(h=h, xhat=xhat, rstd=rstd, logits=logits, lse=lse, labels=labels, shape=tokens.shape,
                              ln_g=ln_g, w_c=w_c)


def classifier_bwd(cache: dict):
    """Returns (dtokens, grads): only the class-token rows of dtokens are non-zero."""
    logits, labels = cache["logits"], cache["labels"]
    Bn = logits.shape[0]
    dl = np.exp(logits - cache["lse"][:, None])
    dl[np.arange(Bn), labels] -= 1.0
    dl /= Bn
    g = dict(w_c=dl.T @ cache["h"], b_c=dl.sum(axis=0))
    dh = dl @ cache["w_c"]
    dcls, g["ln_g"], g["ln_b"] = layer_norm_bwd(dh, cache["xhat"], cache["rstd"], cache["ln_g"])
    dtokens = np.zeros(cache["shape"])
    dtokens[:, 0] = dcls
    return dtokens, g


# ----------------------------------------------------------------------------
# bi-level knapsack scheduling (Alg. 1 and Alg. 2)
# ----------------------------------------------------------------------------
def dp_searching(scores: Sequence[float], weight: int, capacity: int) -> List[int]:
    """0/1 knapsack of one subnet with one common item weight (Alg. 2).

    Fill phase: T[0][w] = 0; T[i][w] = max(T[i-1][w], T[i-1][w-c] + a[i-1]) where
    w >= c, else T[i-1][w].  Backtracking phase: from i = n, w = capacity, while
    both are positive, take item i-1 iff T[i][w] differs from T[i-1][w].
    Returns the 0/1 selection list.
    """
    n, c, C = len(scores), int(weight), int(capacity)
    sel = [0] * n
    if C < 0:
        return sel
    # value table, one row per prefix of the items: row i is row i-1, improved from column c on by taking item i-1
    T = np.zeros((n + 1, C + 1), dtype=np.float64)
    for i, a in enumerate(np.asarray(scores, dtype=np.float64), start=1):
        T[i] = T[i - 1]
        if 0 <= c <= C:
            T[i, c:] = np.maximum(T[i - 1, c:], T[i - 1, :C + 1 - c] + a)
    # an item was taken wherever the value changes between consecutive rows at the remaining capacity
    left = C
    for i in range(n, 0, -1):
        if left <= 0:
            break
        if T[i, left] != T[i - 1, left]:
            sel[i - 1] = 1
            left -= c
    return sel


def knapsack_scheduling(score_full, score_fwd, cost_fwd, cost_bwd, cap_full, cap_fwd) -> np.ndarray:
    """Scheduling table of Alg. 1: uint8 [K, n] with 1 = p_f, 2 = p_o, 3 = p_s.

    Per subnet k: the outer problem (Eq. 4) picks p_f items by backward scores
    with weight c^f_k + c^b_k under cap_full[k]; the inner problem (Eq. 5) picks
    p_o items by forward scores with weight c^f_k under cap_fwd[k]; an item in
    both is p_f, an item in neither is p_s.
    """
    score_full = np.asarray(score_full, dtype=np.float64)
    score_fwd = np.asarray(score_fwd, dtype=np.float64)
    K, n = score_full.shape
    table = np.zeros((K, n), dtype=np.uint8)
    for k in range(K):
        w_b = int(cost_fwd[k]) + int(cost_bwd[k])
        w_f = int(cost_fwd[k])
        t_pf = dp_searching(score_full[k], w_b, int(cap_full[k]))
        t_po = dp_searching(score_fwd[k], w_f, int(cap_fwd[k]))
        pf, po = np.asarray(t_pf, dtype=bool), np.asarray(t_po, dtype=bool)
        table[k] = np.where(pf, OP_FULL, np.where(po, OP_FWD, OP_SKIP))
    return table


# ----------------------------------------------------------------------------
# analytic cost rules (Sec. IV-A)
# ----------------------------------------------------------------------------
def compute_cost_fraction(n_full: int, n_fwd: int, n_skip: int, fwd_share: float = 0.4) -> float:
    """Compute cost relative to all-full: p_o costs fwd_share of p_f, p_s costs nothing."""
    n = n_full + n_fwd + n_skip
    return (n_full + fwd_share * n_fwd) / n


def comm_cost_fraction(n_full: int, n_fwd: int, n_skip: int) -> float:
    """Communication relative to all-full: p_o sends only the forward message (half), p_s none."""
    n = n_full + n_fwd + n_skip
    return (n_full + 0.5 * n_fwd) / n
