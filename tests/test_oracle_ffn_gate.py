"""Pins for the oracle's gated feed-forward slices (no GPU).

With gate_ffn the op code of head h also governs hidden units [h*Dm/H, (h+1)*Dm/H) of the
feed-forward network: the subnet of Sec. II-A.1 (one attention head plus 1/H of the FFN,
Sec. IV-A "Full fine-tuning partition settings").  Checked against things other than the oracle:
  * the all-full mask is the ordinary block (torch fp64 library routines),
  * torch fp64 autograd with .detach() on the forward-only subnets' two contributions,
  * a shortcut subnet equals zeroed W_o columns and zeroed W2 columns of an all-full model,
  * central finite differences with the forward-only contributions held constant,
  * exact zeros in every gradient slice of a subnet that is not p_f, identity for all-shortcut.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import d2ft_inputs as di
from oracle import d2ft_oracle as orc
from test_oracle_block import ALL_FIELDS, MASKS3, draw, relerr, tiny

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def torch_gated_block(wt, ops, x, head_dim, eps=1e-6):
    """Masked block with gated FFN slices in torch fp64 (library routines + autograd)."""
    P = {k: (None if v is None else torch.tensor(np.asarray(v, np.float64), requires_grad=True))
         for k, v in wt.items()}
    xt = torch.tensor(np.asarray(x, np.float64), requires_grad=True)
    D, dh, H = xt.shape[-1], head_dim, len(ops)
    S = P["w1"].shape[0] // H
    live = [h for h, o in enumerate(ops) if o in (FULL, FWD)]
    x1 = xt
    if live:
        u = F.layer_norm(xt, (D,), P["ln1_g"], P["ln1_b"], eps)
        attn = torch.zeros_like(xt)
        for h in live:
            q = F.linear(u, P["w_qkv"][0, h], P["b_qkv"][0, h])
            k = F.linear(u, P["w_qkv"][1, h], P["b_qkv"][1, h])
            v = F.linear(u, P["w_qkv"][2, h], P["b_qkv"][2, h])
            c = F.linear(F.scaled_dot_product_attention(q, k, v), P["w_o"][:, h * dh:(h + 1) * dh])
            attn = attn + (c.detach() if ops[h] == FWD else c)
        if P.get("b_o") is not None:
            attn = attn + P["b_o"]
        x1 = xt + attn
    y = x1
    if live:
        v2 = F.layer_norm(x1, (D,), P["ln2_g"], P["ln2_b"], eps)
        ffn = torch.zeros_like(xt)
        for h in live:
            g = F.gelu(F.linear(v2, P["w1"][h * S:(h + 1) * S], P["b1"][h * S:(h + 1) * S]))
            c = F.linear(g, P["w2"][:, h * S:(h + 1) * S])
            ffn = ffn + (c.detach() if ops[h] == FWD else c)
        if P.get("b2") is not None:
            ffn = ffn + P["b2"]
        y = x1 + ffn
    return y, xt, P


def test_all_full_gated_is_the_ordinary_block():
    w = tiny(heads=3, mlp=48)
    x, wt, dy = draw(w, 21)
    y, cache = orc.block_fwd(wt, [FULL] * 3, x, w.head_dim, gate_ffn=True)
    t = lambda a: torch.tensor(np.asarray(a, np.float64))
    x1 = t(cache["x1"])
    v2 = F.layer_norm(x1, (w.width,), t(wt["ln2_g"]), t(wt["ln2_b"]), 1e-6)
    ref = x1 + F.linear(F.gelu(F.linear(v2, t(wt["w1"]), t(wt["b1"]))), t(wt["w2"]), t(wt["b2"]))
    assert relerr(y, ref.numpy()) < 1e-12
    y0, c0 = orc.block_fwd(wt, [FULL] * 3, x, w.head_dim)
    assert relerr(y, y0) < 1e-13
    dx, g = orc.block_bwd(wt, cache, dy)
    dx0, g0 = orc.block_bwd(wt, c0, dy)
    assert relerr(dx, dx0) < 1e-12
    for k in g0:
        if g0[k] is not None:
            assert relerr(g[k], g0[k]) < 1e-12, k


@pytest.mark.parametrize("ops", MASKS3)
def test_gated_forward_and_backward_match_autograd(ops):
    w = tiny(heads=3, mlp=48)
    x, wt, dy = draw(w, 22)
    y, cache = orc.block_fwd(wt, ops, x, w.head_dim, gate_ffn=True)
    dx, g = orc.block_bwd(wt, cache, dy)
    ref, xt, P = torch_gated_block(wt, ops, x, w.head_dim)
    assert relerr(y, ref.detach().numpy()) < 1e-12
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


def test_all_shortcut_gated_block_is_the_identity():
    w = tiny(heads=3, mlp=48)
    x, wt, dy = draw(w, 23)
    y, cache = orc.block_fwd(wt, [SKIP] * 3, x, w.head_dim, gate_ffn=True)
    assert np.array_equal(y, x)                      # no bias of either side is applied
    dx, g = orc.block_bwd(wt, cache, dy)
    assert np.array_equal(dx, dy)
    for k, v in g.items():
        if v is not None:
            assert np.all(v == 0.0), k


@pytest.mark.parametrize("ops", [(FULL, SKIP, FULL), (SKIP, FULL, FWD), (FWD, SKIP, SKIP)])
def test_shortcut_subnet_equals_zeroed_projection_columns(ops):
    """A shortcut subnet == all-full model with that head's W_o columns and its slice's W2 columns zeroed."""
    w = tiny(heads=3, mlp=48)
    x, wt, _ = draw(w, 24)
    S = w.mlp_hidden // w.heads
    y, _ = orc.block_fwd(wt, ops, x, w.head_dim, gate_ffn=True)
    wz = dict(wt)
    wz["w_o"], wz["w2"] = wt["w_o"].copy(), wt["w2"].copy()
    for h, o in enumerate(ops):
        if o == SKIP:
            wz["w_o"][:, h * w.head_dim:(h + 1) * w.head_dim] = 0.0
            wz["w2"][:, h * S:(h + 1) * S] = 0.0
    y2, _ = orc.block_fwd(wz, [FULL] * 3, x, w.head_dim)          # ungated path of the oracle
    assert relerr(y, y2) < 1e-13


@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP), (SKIP, FWD, FULL), (FWD, FULL, FWD)])
def test_gated_non_full_subnets_get_exactly_zero_gradients(ops):
    w = tiny(heads=3, mlp=48)
    x, wt, dy = draw(w, 25)
    S = w.mlp_hidden // w.heads
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim, gate_ffn=True)
    _, g = orc.block_bwd(wt, cache, dy)
    for h, o in enumerate(ops):
        for s in (g["w1"][h * S:(h + 1) * S], g["b1"][h * S:(h + 1) * S], g["w2"][:, h * S:(h + 1) * S]):
            if o == FULL:
                assert np.abs(s).max() > 0.0
            else:
                assert np.all(s == 0.0) and not np.any(np.signbit(s))


def test_gated_no_full_subnet_passes_the_gradient_through():
    w = tiny(heads=3, mlp=48)
    x, wt, dy = draw(w, 26)
    _, cache = orc.block_fwd(wt, (FWD, SKIP, FWD), x, w.head_dim, gate_ffn=True)
    dx, g = orc.block_bwd(wt, cache, dy)
    assert np.array_equal(dx, dy)                    # residual route only (Sec. II-A.2)
    s = dy.reshape(-1, w.width).sum(0)
    assert relerr(g["b_o"], s) < 1e-12 and relerr(g["b2"], s) < 1e-12
    for k in ("w_qkv", "b_qkv", "w_o", "w1", "b1", "w2", "ln1_g", "ln1_b", "ln2_g", "ln2_b"):
        assert np.all(g[k] == 0.0), k


@pytest.mark.parametrize("ops", [(FULL, FULL), (FULL, SKIP), (FULL, FWD), (FWD, FULL)])
def test_gated_finite_differences(ops):
    """Central differences of <dy, y(theta)> with the forward-only subnets' two terms held constant."""
    w = di.Workload("fd", 1, 5, 8, 2, 4, 16, 1, "f32")
    x, wt, dy = draw(w, 27)
    S = w.mlp_hidden // w.heads
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim, gate_ffn=True)
    dx, g = orc.block_bwd(wt, cache, dy)
    a_const, f_const = np.zeros_like(x), np.zeros_like(x)
    for h, o in enumerate(ops):
        if o == FWD:
            a_const = a_const + cache["heads"][h]["contrib"]
            f_const = f_const + cache["slices"][h]["g"] @ wt["w2"][:, h * S:(h + 1) * S].T
    ops_fd = [SKIP if o == FWD else o for o in ops]

    def f(wp, xp):
        y, _ = orc.block_fwd(wp, ops_fd, xp, w.head_dim, attn_const=a_const, gate_ffn=True, ffn_const=f_const)
        return float((y * dy).sum())

    rng = np.random.default_rng(127)
    eps = 1e-6
    for name in ALL_FIELDS:
        base = x if name == "x" else wt[name]
        ana = dx if name == "x" else g[name]
        for fi in rng.choice(base.size, size=min(6, base.size), replace=False):
            idx = np.unravel_index(fi, base.shape)

            def at(delta):
                if name == "x":
                    xp = x.copy(); xp[idx] += delta
                    return f(wt, xp)
                wp = dict(wt); wp[name] = wt[name].copy(); wp[name][idx] += delta
                return f(wp, x)
            num = (at(eps) - at(-eps)) / (2 * eps)
            scale = max(1.0, abs(num), np.abs(ana).max())
            assert abs(num - ana[idx]) <= 2e-6 * scale, (name, idx, num, ana[idx])


def test_gated_stack_matches_torch_chain():
    w = di.Workload("stack", 2, 6, 16, 2, 8, 24, 3, "f32")
    rng = np.random.default_rng(28)
    x = rng.standard_normal((w.batch, w.tokens, w.width))
    weights = [{k: (None if v is None else v.astype(np.float64) * 8) for k, v in di.draw_block_weights(rng, w).items()}
               for _ in range(w.blocks)]
    ops = np.array([[FULL, FWD], [SKIP, FULL], [SKIP, SKIP]], dtype=np.uint8)
    y, _ = orc.stack_fwd(weights, ops, x, w.head_dim, gate_ffn=True)
    h = torch.tensor(x)
    for l in range(w.blocks):
        h, _, _ = torch_gated_block(weights[l], ops[l], h.detach().numpy(), w.head_dim)
    assert relerr(y, h.detach().numpy()) < 1e-11
