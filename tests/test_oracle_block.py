"""Pins for the CPU oracle's block forward / backward (no GPU).

The oracle is checked against things other than itself:
  * torch fp64 library routines (scaled_dot_product_attention,
    multi_head_attention_forward, layer_norm, linear, gelu) for the all-full
    mask, which the paper defines as standard fine-tuning (Sec. II-A.2, p_f),
  * torch fp64 autograd with .detach() on forward-only heads for the
    stop-gradient reading of p_o,
  * central finite differences of the forward,
  * structural invariants: all-shortcut leaves only the residual + MLP path,
    a shortcut head equals a zeroed output-projection slice, forward-only and
    shortcut heads get exactly zero gradients.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import d2ft_inputs as di
from oracle import d2ft_oracle as orc

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def tiny(heads=3, lora_rank=0, tokens=7, batch=2, width=24, head_dim=8, mlp=40, lora_b_zero=False):
    return di.Workload("tiny", batch, tokens, width, heads, head_dim, mlp, 1, "f32",
                       lora_rank=lora_rank, lora_b_zero=lora_b_zero)


def draw(w, seed=0, big_weights=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((w.batch, w.tokens, w.width))
    wt = di.draw_block_weights(rng, w)
    if big_weights:   # make every path numerically visible on tiny shapes
        wt = {k: (None if v is None else (v.astype(np.float64) * (1.0 if k.startswith("ln") and k.endswith("_g") else 10.0)))
              for k, v in wt.items()}
        wt["ln1_g"] = wt["ln1_g"] + 0.3 * rng.standard_normal(w.width)
        wt["ln2_g"] = wt["ln2_g"] + 0.3 * rng.standard_normal(w.width)
    dy = rng.standard_normal((w.batch, w.tokens, w.width))
    return x, wt, dy


# ---------------------------------------------------------------------------
# an independent torch fp64 implementation (library routines + autograd)
# ---------------------------------------------------------------------------
def torch_block(wt, ops, x, head_dim, eps=1e-6, lora_scale=1.0):
    """Masked block in torch fp64.  Returns (y, x1, params) with autograd graph."""
    P = {k: (None if v is None else torch.tensor(np.asarray(v, np.float64), requires_grad=True))
         for k, v in wt.items()}
    xt = torch.tensor(np.asarray(x, np.float64), requires_grad=True)
    B, T, D = xt.shape
    dh = head_dim
    live = [h for h, o in enumerate(ops) if o in (FULL, FWD)]
    attn = torch.zeros_like(xt)
    if live:
        u = F.layer_norm(xt, (D,), P["ln1_g"], P["ln1_b"], eps)
        for h in live:
            wq, wk, wv = P["w_qkv"][0, h], P["w_qkv"][1, h], P["w_qkv"][2, h]
            if P.get("lora_a_q") is not None:
                wq = wq + lora_scale * P["lora_b_q"][h] @ P["lora_a_q"][h]
                wv = wv + lora_scale * P["lora_b_v"][h] @ P["lora_a_v"][h]
            q = F.linear(u, wq, P["b_qkv"][0, h])
            k = F.linear(u, wk, P["b_qkv"][1, h])
            v = F.linear(u, wv, P["b_qkv"][2, h])
            o = F.scaled_dot_product_attention(q, k, v)            # scale 1/sqrt(dh), no mask
            c = F.linear(o, P["w_o"][:, h * dh:(h + 1) * dh])
            if ops[h] == FWD:
                c = c.detach()
            attn = attn + c
        if P.get("b_o") is not None:
            attn = attn + P["b_o"]
    x1 = xt + attn
    v2 = F.layer_norm(x1, (D,), P["ln2_g"], P["ln2_b"], eps)
    y = x1 + F.linear(F.gelu(F.linear(v2, P["w1"], P["b1"])), P["w2"], P["b2"])
    return y, xt, P


def relerr(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.abs(b).max()
    return np.abs(a - b).max() / (den if den > 0 else 1.0)


MASKS3 = [(FULL, FULL, FULL), (FULL, FWD, SKIP), (SKIP, FULL, FWD), (FWD, FWD, FULL),
          (SKIP, SKIP, FULL), (FWD, FWD, FWD), (SKIP, SKIP, SKIP), (FWD, SKIP, SKIP)]


# ---------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------
def test_all_full_equals_library_multi_head_attention():
    """All-full mask == standard pre-LN block built on torch's own MHA routine."""
    w = tiny(heads=3)
    x, wt, _ = draw(w, 1)
    y, cache = orc.block_fwd(wt, [FULL] * 3, x, w.head_dim)
    D, H, dh = w.width, w.heads, w.head_dim
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    xt = t(x)
    u = F.layer_norm(xt, (D,), t(wt["ln1_g"]), t(wt["ln1_b"]), 1e-6)
    a, _ = F.multi_head_attention_forward(
        u.transpose(0, 1), u.transpose(0, 1), u.transpose(0, 1), D, H,
        t(wt["w_qkv"]).reshape(3 * H * dh, D), t(wt["b_qkv"]).reshape(-1), None, None, False, 0.0,
        t(wt["w_o"]), t(wt["b_o"]), need_weights=False)
    x1 = xt + a.transpose(0, 1)
    v2 = F.layer_norm(x1, (D,), t(wt["ln2_g"]), t(wt["ln2_b"]), 1e-6)
    ref = x1 + F.linear(F.gelu(F.linear(v2, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))
    assert relerr(cache["x1"], x1.numpy()) < 1e-12
    assert relerr(y, ref.numpy()) < 1e-12


@pytest.mark.parametrize("ops", MASKS3)
def test_forward_matches_torch_for_any_mask(ops):
    w = tiny(heads=3)
    x, wt, _ = draw(w, 2)
    y, _ = orc.block_fwd(wt, ops, x, w.head_dim)
    ref, _, _ = torch_block(wt, ops, x, w.head_dim)
    assert relerr(y, ref.detach().numpy()) < 1e-12


def test_all_skip_leaves_residual_plus_mlp():
    w = tiny(heads=3)
    x, wt, _ = draw(w, 3)
    y, cache = orc.block_fwd(wt, [SKIP] * 3, x, w.head_dim)
    assert np.array_equal(cache["x1"], x)             # bitwise: attention side untouched, no b_o
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    v2 = F.layer_norm(t(x), (w.width,), t(wt["ln2_g"]), t(wt["ln2_b"]), 1e-6)
    ref = t(x) + F.linear(F.gelu(F.linear(v2, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))
    assert relerr(y, ref.numpy()) < 1e-12


@pytest.mark.parametrize("ops", [(FULL, SKIP, FULL), (SKIP, FULL, FWD), (FWD, SKIP, SKIP)])
def test_skipped_head_equals_zeroed_output_projection(ops):
    """Forward with a shortcut head == all-live forward with that head's W_o columns zeroed."""
    w = tiny(heads=3)
    x, wt, _ = draw(w, 4)
    y, _ = orc.block_fwd(wt, ops, x, w.head_dim)
    wz = dict(wt)
    wz["w_o"] = wt["w_o"].copy()
    for h, o in enumerate(ops):
        if o == SKIP:
            wz["w_o"][:, h * w.head_dim:(h + 1) * w.head_dim] = 0.0
    y2, _ = orc.block_fwd(wz, [FULL] * 3, x, w.head_dim)
    assert relerr(y, y2) < 1e-13


def test_null_biases():
    w = tiny(heads=2)
    x, wt, dy = draw(w, 5)
    wt["b_o"] = None
    wt["b2"] = None
    ops = (FULL, FWD)
    y, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    ref, xt, P = torch_block(wt, ops, x, w.head_dim)
    assert relerr(y, ref.detach().numpy()) < 1e-12
    dx, g = orc.block_bwd(wt, cache, dy)
    ref.backward(torch.tensor(dy))
    assert relerr(dx, xt.grad.numpy()) < 1e-11
    assert g["b_o"] is None and g["b2"] is None


# ---------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------
def _check_against_autograd(w, ops, seed, lora_scale=1.0):
    x, wt, dy = draw(w, seed)
    y, cache = orc.block_fwd(wt, ops, x, w.head_dim, lora_scale=lora_scale)
    dx, g = orc.block_bwd(wt, cache, dy)
    ref, xt, P = torch_block(wt, ops, x, w.head_dim, lora_scale=lora_scale)
    ref.backward(torch.tensor(dy))
    assert relerr(dx, xt.grad.numpy()) < 1e-11
    for k, p in P.items():
        if p is None:
            continue
        gr = np.zeros(p.shape) if p.grad is None else p.grad.numpy()
        if np.abs(gr).max() == 0.0:
            assert np.all(g[k] == 0.0), k
        else:
            assert relerr(g[k], gr) < 1e-10, k
    return g


@pytest.mark.parametrize("ops", MASKS3)
def test_backward_matches_autograd_with_detached_forward_only_heads(ops):
    _check_against_autograd(tiny(heads=3), ops, 6)


@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP), (FULL, FULL, FULL), (FWD, SKIP, FULL)])
def test_lora_backward_matches_autograd(ops):
    _check_against_autograd(tiny(heads=3, lora_rank=2), ops, 7, lora_scale=0.7)


@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP), (SKIP, FWD, FULL), (FWD, FULL, FWD)])
def test_non_full_heads_get_exactly_zero_gradients(ops):
    w = tiny(heads=3, lora_rank=2)
    x, wt, dy = draw(w, 8)
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    _, g = orc.block_bwd(wt, cache, dy)
    dh = w.head_dim
    for h, o in enumerate(ops):
        slices = [g["w_qkv"][:, h], g["b_qkv"][:, h], g["w_o"][:, h * dh:(h + 1) * dh],
                  g["lora_a_q"][h], g["lora_a_v"][h], g["lora_b_q"][h], g["lora_b_v"][h]]
        for s in slices:
            if o == FULL:
                assert np.abs(s).max() > 0.0
            else:
                assert np.all(s == 0.0) and not np.any(np.signbit(s))


def test_key_bias_gradient_vanishes_and_value_bias_gradient_is_the_sum_of_dO():
    """Two closed forms of softmax attention (Sec. II-A.2, the p_f backward).  A shift of every key of a head
    by the same vector moves all scores of a query by the same amount, which the softmax does not see, so the
    gradient of the key bias is zero.  The rows of the probability matrix sum to one, so the gradient of the
    value bias is the column sum of the gradient that reaches the head's output."""
    w = tiny(heads=3)
    x, wt, dy = draw(w, 21)
    ops = (FULL, FWD, FULL)
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    _, g = orc.block_bwd(wt, cache, dy)
    scale = np.abs(g["b_qkv"]).max()
    assert scale > 0.0
    dh = w.head_dim
    # dO = dx1 W_o[:, head]: rebuilt here from the out-projection bias gradient's operand, dx1 = sum of dy routes
    # (taken through autograd, which knows neither identity)
    ref, xt, P = torch_block(wt, ops, x, w.head_dim)
    ref.backward(torch.tensor(dy))
    gb = P["b_qkv"].grad.numpy()
    for h, o in enumerate(ops):
        if o != FULL:
            continue
        assert np.abs(g["b_qkv"][1, h]).max() <= 1e-12 * scale        # key plane
        assert np.abs(gb[1, h]).max() <= 1e-12 * scale
        assert relerr(g["b_qkv"][2, h], gb[2, h]) < 1e-10             # value plane against autograd
    # the value plane is also W_o^T applied to the out-projection bias gradient, head by head
    wo = wt["w_o"]
    for h, o in enumerate(ops):
        if o == FULL:
            assert relerr(g["b_qkv"][2, h], g["b_o"] @ wo[:, h * dh:(h + 1) * dh]) < 1e-10


def test_no_full_heads_gives_residual_and_mlp_gradient_only():
    w = tiny(heads=3)
    x, wt, dy = draw(w, 9)
    ops = (FWD, SKIP, FWD)
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    dx, g = orc.block_bwd(wt, cache, dy)
    # dx must equal the gradient of x1 -> y alone (identity on the attention side)
    x1 = torch.tensor(cache["x1"], requires_grad=True)
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    v2 = F.layer_norm(x1, (w.width,), t(wt["ln2_g"]), t(wt["ln2_b"]), 1e-6)
    y = x1 + F.linear(F.gelu(F.linear(v2, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))
    y.backward(torch.tensor(dy))
    assert relerr(dx, x1.grad.numpy()) < 1e-11
    for k in ("w_qkv", "b_qkv", "w_o", "ln1_g", "ln1_b"):
        assert np.all(g[k] == 0.0)
    assert relerr(g["b_o"], x1.grad.numpy().reshape(-1, w.width).sum(0)) < 1e-11


def _fd_check(w, ops, seed, fields, lora_scale=1.0, n_probe=6, h=1e-6, tol=2e-6):
    """Central differences of f(theta) = <dy, y(theta)> with forward-only heads held constant."""
    x, wt, dy = draw(w, seed)
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim, lora_scale=lora_scale)
    dx, g = orc.block_bwd(wt, cache, dy)
    # constant part: the forward-only heads' contribution at the unperturbed point
    const = np.zeros_like(x)
    for hh, o in enumerate(ops):
        if o == FWD:
            const = const + cache["heads"][hh]["contrib"]
    ops_fd = [SKIP if o == FWD else o for o in ops]
    assert any(o == FULL for o in ops)   # keeps b_o applied in the perturbed model too

    def f(wp, xp):
        y, _ = orc.block_fwd(wp, ops_fd, xp, w.head_dim, lora_scale=lora_scale, attn_const=const)
        return float((y * dy).sum())

    rng = np.random.default_rng(seed + 100)
    for name in fields:
        base = x if name == "x" else wt[name]
        ana = dx if name == "x" else g[name]
        flat_idx = rng.choice(base.size, size=min(n_probe, base.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, base.shape)
            def at(delta):
                if name == "x":
                    xp = x.copy(); xp[idx] += delta
                    return f(wt, xp)
                wp = dict(wt); wp[name] = wt[name].copy(); wp[name][idx] += delta
                return f(wp, x)
            num = (at(h) - at(-h)) / (2 * h)
            scale = max(1.0, abs(num), np.abs(ana).max())
            assert abs(num - ana[idx]) <= tol * scale, (name, idx, num, ana[idx])


ALL_FIELDS = ["x", "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"]


@pytest.mark.parametrize("ops", [(FULL, FULL), (FULL, SKIP), (FULL, FWD), (FWD, FULL)])
def test_finite_differences(ops):
    w = di.Workload("fd", 1, 5, 8, 2, 4, 16, 1, "f32")
    _fd_check(w, ops, 10, ALL_FIELDS)


def test_finite_differences_lora():
    w = di.Workload("fd", 1, 5, 8, 3, 4, 16, 1, "f32", lora_rank=2, lora_b_zero=False)
    _fd_check(w, (FULL, FWD, FULL), 11, ALL_FIELDS + ["lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"],
              lora_scale=1.3)


def test_lora_zero_b_equals_base_and_gives_zero_a_gradient():
    w = tiny(heads=2, lora_rank=2, lora_b_zero=True)
    x, wt, dy = draw(w, 12)
    assert np.all(wt["lora_b_q"] == 0) and np.all(wt["lora_b_v"] == 0)
    ops = (FULL, FULL)
    y, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    base = {k: (None if k.startswith("lora") else v) for k, v in wt.items()}
    y0, _ = orc.block_fwd(base, ops, x, w.head_dim)
    assert np.array_equal(y, y0)
    _, g = orc.block_bwd(wt, cache, dy)
    assert np.all(g["lora_a_q"] == 0.0) and np.all(g["lora_a_v"] == 0.0)
    assert np.abs(g["lora_b_q"]).max() > 0 and np.abs(g["lora_b_v"]).max() > 0


def test_stack_matches_torch_chain():
    w = di.Workload("stack", 2, 6, 16, 2, 8, 24, 3, "f32")
    rng = np.random.default_rng(13)
    x = rng.standard_normal((w.batch, w.tokens, w.width))
    weights = [{k: (None if v is None else v.astype(np.float64) * 8) for k, v in di.draw_block_weights(rng, w).items()}
               for _ in range(w.blocks)]
    dy = rng.standard_normal(x.shape)
    ops = np.array([[FULL, FWD], [SKIP, FULL], [FWD, SKIP]], dtype=np.uint8)
    y, caches = orc.stack_fwd(weights, ops, x, w.head_dim)
    dx, grads = orc.stack_bwd(weights, caches, dy)
    # torch chain
    h = torch.tensor(x, requires_grad=True)
    cur, Ps = h, []
    for l in range(w.blocks):
        yb, xin, P = torch_block(weights[l], list(ops[l]), cur.detach().numpy(), w.head_dim)
        # rebuild on the running graph: feed cur instead of a fresh leaf
        Ps.append((yb, xin, P))
        cur = yb
    assert relerr(y, cur.detach().numpy()) < 1e-12
    # backward block by block through the torch graphs
    d = torch.tensor(dy)
    for l in range(w.blocks - 1, -1, -1):
        yb, xin, P = Ps[l]
        yb.backward(d)
        d = xin.grad
        assert relerr(grads[l]["w1"], P["w1"].grad.numpy()) < 1e-10
    assert relerr(dx, d.numpy()) < 1e-10
