"""Pins for the oracle's contribution scores (Sec. II-B: Fisher information = sum of squared gradient
entries of a subnet, weight magnitude = sum of absolute weights).  No GPU.

Checked against things other than the oracle's own expression: element counts derived from the shapes
with constant-valued subnets, torch norms over slices taken by a different indexing route (reshape +
unbind instead of the oracle's slicing), permutation of two heads, additivity over fields, and the
Fisher score of a real backward pass against torch autograd's per-head gradient norms.
"""
import numpy as np
import pytest
import torch

import d2ft_inputs as di
from oracle import d2ft_oracle as orc
from test_oracle_block import draw, tiny, torch_block

FULL = di.OP_FULL


def counts(w, gate):
    """Entries owned by one head, from the shapes alone."""
    D, dh, r = w.width, w.head_dim, w.lora_rank
    n = 3 * dh * D + 3 * dh + D * dh
    if r:
        n += 2 * r * D + 2 * dh * r
    if gate:
        S = w.mlp_hidden // w.heads
        n += S * D + S + D * S
    return n


@pytest.mark.parametrize("gate", [False, True])
@pytest.mark.parametrize("rank", [0, 2])
def test_constant_subnets_give_count_times_value(gate, rank):
    w = tiny(heads=3, lora_rank=rank, mlp=48)
    _, wt, _ = draw(w, 41)
    S = w.mlp_hidden // w.heads
    vals = [0.5, -2.0, 3.0]
    t = {k: (None if v is None else np.zeros_like(v, dtype=np.float64)) for k, v in wt.items()}
    for h, v in enumerate(vals):
        t["w_qkv"][:, h] = v; t["b_qkv"][:, h] = v
        t["w_o"][:, h * w.head_dim:(h + 1) * w.head_dim] = v
        for k in ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"):
            if t.get(k) is not None:
                t[k][h] = v
        t["w1"][h * S:(h + 1) * S] = v; t["b1"][h * S:(h + 1) * S] = v; t["w2"][:, h * S:(h + 1) * S] = v
    # tensors that belong to no single subnet must not count
    for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "b_o", "b2"):
        t[k] = np.full_like(t[k], 7.0)
    n = counts(w, gate)
    fis = orc.subnet_scores(t, w.heads, w.head_dim, "fisher", gate_ffn=gate)
    mag = orc.subnet_scores(t, w.heads, w.head_dim, "magnitude", gate_ffn=gate)
    assert np.allclose(fis, [n * v * v for v in vals], rtol=1e-14)
    assert np.allclose(mag, [n * abs(v) for v in vals], rtol=1e-14)


@pytest.mark.parametrize("gate", [False, True])
def test_scores_match_torch_norms_over_reshaped_views(gate):
    w = tiny(heads=3, lora_rank=2, mlp=48)
    _, wt, _ = draw(w, 42)
    H, dh, D = w.heads, w.head_dim, w.width
    S = w.mlp_hidden // H
    T = {k: (None if v is None else torch.tensor(np.asarray(v, np.float64))) for k, v in wt.items()}
    fis = orc.subnet_scores(wt, H, dh, "fisher", gate_ffn=gate)
    mag = orc.subnet_scores(wt, H, dh, "magnitude", gate_ffn=gate)
    for h in range(H):
        pieces = [T["w_qkv"].permute(1, 0, 2, 3).unbind(0)[h], T["b_qkv"].permute(1, 0, 2).unbind(0)[h],
                  T["w_o"].reshape(D, H, dh).unbind(1)[h]]
        pieces += [T[k].unbind(0)[h] for k in ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v")]
        if gate:
            pieces += [T["w1"].reshape(H, S, D).unbind(0)[h], T["b1"].reshape(H, S).unbind(0)[h],
                       T["w2"].reshape(D, H, S).unbind(1)[h]]
        l2 = sum(float(torch.linalg.vector_norm(p, 2)) ** 2 for p in pieces)
        l1 = sum(float(torch.linalg.vector_norm(p, 1)) for p in pieces)
        assert abs(fis[h] - l2) <= 1e-12 * l2 and abs(mag[h] - l1) <= 1e-12 * l1


def test_swapping_two_heads_swaps_their_scores():
    w = tiny(heads=3, mlp=48)
    _, wt, _ = draw(w, 43)
    S, dh = w.mlp_hidden // w.heads, w.head_dim
    sw = {k: (None if v is None else np.array(v, dtype=np.float64)) for k, v in wt.items()}
    a, b = 0, 2
    for k in ("w_qkv", "b_qkv"):
        sw[k][:, [a, b]] = sw[k][:, [b, a]]
    cols = lambda m, h, n: m[:, h * n:(h + 1) * n].copy()
    wa, wb = cols(sw["w_o"], a, dh), cols(sw["w_o"], b, dh)
    sw["w_o"][:, a * dh:(a + 1) * dh], sw["w_o"][:, b * dh:(b + 1) * dh] = wb, wa
    for k in ("w1", "b1"):
        ra, rb = sw[k][a * S:(a + 1) * S].copy(), sw[k][b * S:(b + 1) * S].copy()
        sw[k][a * S:(a + 1) * S], sw[k][b * S:(b + 1) * S] = rb, ra
    ca, cb = cols(sw["w2"], a, S), cols(sw["w2"], b, S)
    sw["w2"][:, a * S:(a + 1) * S], sw["w2"][:, b * S:(b + 1) * S] = cb, ca
    for kind in ("fisher", "magnitude"):
        s0 = orc.subnet_scores(wt, w.heads, dh, kind, gate_ffn=True)
        s1 = orc.subnet_scores(sw, w.heads, dh, kind, gate_ffn=True)
        assert np.allclose(s1, s0[[2, 1, 0]], rtol=1e-13)


def test_none_fields_are_skipped_and_scores_add_over_fields():
    w = tiny(heads=2, mlp=32)
    _, wt, _ = draw(w, 44)
    full = orc.subnet_scores(wt, w.heads, w.head_dim, "fisher")
    acc = np.zeros(w.heads)
    for k in ("w_qkv", "b_qkv", "w_o"):
        only = {kk: (v if kk == k else None) for kk, v in wt.items()}
        acc += orc.subnet_scores(only, w.heads, w.head_dim, "fisher")
    assert np.allclose(acc, full, rtol=1e-13)


def test_fisher_score_of_a_backward_pass_matches_autograd_gradient_norms():
    w = tiny(heads=3)
    x, wt, dy = draw(w, 45)
    ops = [FULL] * 3
    _, cache = orc.block_fwd(wt, ops, x, w.head_dim)
    _, g = orc.block_bwd(wt, cache, dy)
    fis = orc.subnet_scores(g, w.heads, w.head_dim, "fisher")
    ref, _, P = torch_block(wt, ops, x, w.head_dim)
    ref.backward(torch.tensor(dy))
    dh = w.head_dim
    for h in range(w.heads):
        tot = float((P["w_qkv"].grad[:, h] ** 2).sum() + (P["b_qkv"].grad[:, h] ** 2).sum()
                    + (P["w_o"].grad[:, h * dh:(h + 1) * dh] ** 2).sum())
        assert abs(fis[h] - tot) <= 1e-9 * tot
