"""Pins for the oracle's SGD-with-momentum step on p_f subnets (Sec. IV-A names the optimizer).  No GPU.

  * torch.optim.SGD (library routine) run on parameters that hold exactly the selected slices, several
    steps with momentum and weight decay;
  * slices of subnets that were not p_f, and their momentum, stay bit for bit;
  * one step from zero momentum is w - lr*(g + wd*w) (closed form).
"""
import numpy as np
import pytest
import torch

import d2ft_inputs as di
from oracle import d2ft_oracle as orc
from test_oracle_block import draw, tiny

SHARED = ("ln1_g", "ln1_b", "b_o", "ln2_g", "ln2_b", "b2")


def owner_map(k, shape, w, gate):
    """Head that owns each element of tensor k (-1: shared by all subnets), built from the layout of
    Sec. II-A.1 by broadcasting a head index over a reshaped view - not from the oracle's own slicing."""
    H, dh = w.heads, w.head_dim
    heads = np.arange(H)
    if k == "w_qkv":      # [3][H][dh][D]
        return np.broadcast_to(heads[None, :, None, None], shape).copy()
    if k == "b_qkv":      # [3][H][dh]
        return np.broadcast_to(heads[None, :, None], shape).copy()
    if k == "w_o":        # [D][H*dh]: column h*dh + d belongs to head h
        return np.broadcast_to(heads[None, :, None], (shape[0], H, dh)).reshape(shape).copy()
    if k.startswith("lora_"):   # [H][...]
        return np.broadcast_to(heads.reshape((H,) + (1,) * (len(shape) - 1)), shape).copy()
    if gate and k in ("w1", "b1"):   # rows (hidden units) in H contiguous groups
        S = shape[0] // H
        return np.broadcast_to(np.repeat(heads, S).reshape((shape[0],) + (1,) * (len(shape) - 1)), shape).copy()
    if gate and k == "w2":           # [D][Dm]: columns in H contiguous groups
        S = shape[1] // H
        return np.broadcast_to(np.repeat(heads, S)[None, :], shape).copy()
    return np.full(shape, -1)


@pytest.mark.parametrize("gate", [False, True])
def test_matches_torch_sgd_on_the_selected_slices(gate):
    w = tiny(heads=3, lora_rank=2, mlp=48)
    rng = np.random.default_rng(81)
    _, wt, _ = draw(w, 81)
    wt = {k: (None if a is None else np.asarray(a, np.float64)) for k, a in wt.items()}
    vt = {k: (None if a is None else np.zeros_like(a)) for k, a in wt.items()}
    own = {k: owner_map(k, a.shape, w, gate) for k, a in wt.items() if a is not None}
    w0 = {k: a.copy() for k, a in wt.items()}
    updated_seq = [[True, False, True], [False, False, True], [True, True, False]]
    lr, mu, wd = 0.05, 0.9, 0.01
    # torch side: one flat parameter per (tensor, owner) actually trained, gathered by boolean masks
    params = {}
    for k, a in wt.items():
        for tag in np.unique(own[k]):
            params[(k, int(tag))] = torch.nn.Parameter(torch.tensor(a[own[k] == tag].copy()))
    # one optimizer per region so that a region skipped in a step keeps its momentum untouched
    opts = {key: torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd) for key, p in params.items()}
    for step, updated in enumerate(updated_seq):
        g = {k: rng.standard_normal(a.shape) for k, a in wt.items()}
        wt, vt = orc.sgd_momentum_step(wt, g, vt, updated, w.head_dim, lr, mu, wd, gate_ffn=gate)
        for (k, tag), p in params.items():
            if tag >= 0 and not updated[tag]:
                continue
            p.grad = torch.tensor(g[k][own[k] == tag].copy())
            opts[(k, tag)].step()
    for (k, tag), p in params.items():
        assert np.allclose(wt[k][own[k] == tag], p.detach().numpy(), rtol=1e-12, atol=1e-14), (k, tag)
    # every per-head tensor has all three owners, and the feed-forward tensors are owned only when gated
    for k in ("w_qkv", "b_qkv", "w_o", "lora_a_q", "lora_b_v"):
        assert sorted(np.unique(own[k])) == [0, 1, 2]
    for k in ("w1", "b1", "w2"):
        assert sorted(np.unique(own[k])) == ([0, 1, 2] if gate else [-1])
    for k in wt:
        assert not np.array_equal(wt[k], w0[k]), k


def test_skipped_subnets_keep_weights_and_momentum_bitwise():
    w = tiny(heads=3, mlp=48)
    rng = np.random.default_rng(82)
    _, wt, _ = draw(w, 82)
    vt = {k: (None if a is None else rng.standard_normal(a.shape)) for k, a in wt.items()}
    g = {k: (None if a is None else rng.standard_normal(a.shape)) for k, a in wt.items()}
    w2, v2 = orc.sgd_momentum_step(wt, g, vt, [False, True, False], w.head_dim, 0.1, 0.9, 0.0, gate_ffn=True)
    n_owned = 0
    for k, a in wt.items():
        if a is None:
            continue
        own = owner_map(k, np.shape(a), w, True)
        if (own < 0).all():
            continue
        n_owned += 1
        a64 = np.asarray(a, np.float64)
        for h in (0, 2):
            r = own == h
            assert np.array_equal(w2[k][r], a64[r]) and np.array_equal(v2[k][r], vt[k][r]), k
        r = own == 1
        # every element of the trained subnet moves (lr * v is never exactly zero for these draws)
        assert np.all(w2[k][r] != a64[r]) and np.all(v2[k][r] != vt[k][r]), k
    assert n_owned == 6   # w_qkv, b_qkv, w_o, w1, b1, w2
    for k in SHARED:
        assert not np.array_equal(w2[k], np.asarray(wt[k], np.float64)), k     # shared tensors always move


def test_first_step_closed_form_and_untrained_fields():
    w = tiny(heads=2)
    rng = np.random.default_rng(83)
    _, wt, _ = draw(w, 83)
    vt = {k: (None if a is None else np.zeros_like(a, dtype=np.float64)) for k, a in wt.items()}
    g = {k: (rng.standard_normal(a.shape) if k in ("w_qkv", "w1") else None) for k, a in wt.items()}
    w2, v2 = orc.sgd_momentum_step(wt, g, vt, [True, True], w.head_dim, 0.3, 0.5, 0.2)
    for k in ("w_qkv", "w1"):
        a = np.asarray(wt[k], np.float64)
        assert np.allclose(w2[k], a - 0.3 * (g[k] + 0.2 * a), rtol=1e-14)
    for k in ("w_o", "b_qkv", "w2", "b_o"):
        assert np.array_equal(w2[k], np.asarray(wt[k], np.float64)) and np.all(v2[k] == 0.0)
