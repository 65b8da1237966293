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


def slices_of(k, a, h, w, gate):
    return orc._head_slices(k, a, h, w.heads, w.head_dim, gate)


@pytest.mark.parametrize("gate", [False, True])
def test_matches_torch_sgd_on_the_selected_slices(gate):
    w = tiny(heads=3, lora_rank=2, mlp=48)
    rng = np.random.default_rng(81)
    _, wt, _ = draw(w, 81)
    wt = {k: (None if a is None else np.asarray(a, np.float64)) for k, a in wt.items()}
    vt = {k: (None if a is None else np.zeros_like(a)) for k, a in wt.items()}
    updated_seq = [[True, False, True], [False, False, True], [True, True, False]]
    lr, mu, wd = 0.05, 0.9, 0.01
    # torch side: one parameter per (tensor, region) actually trained, gathered by numpy indexing
    params = {}
    def region_list(k, a):
        if slices_of(k, a, 0, w, gate) is None:
            return [("all", (slice(None),))]
        return [(h, slices_of(k, a, h, w, gate)) for h in range(w.heads)]
    for k, a in wt.items():
        for tag, r in region_list(k, a):
            params[(k, tag)] = torch.nn.Parameter(torch.tensor(a[r].copy()))
    # one optimizer per region so that a region skipped in a step keeps its momentum untouched
    opts = {key: torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd) for key, p in params.items()}
    for step, updated in enumerate(updated_seq):
        g = {k: rng.standard_normal(a.shape) for k, a in wt.items()}
        wt, vt = orc.sgd_momentum_step(wt, g, vt, updated, w.head_dim, lr, mu, wd, gate_ffn=gate)
        for (k, tag), p in params.items():
            if tag != "all" and not updated[tag]:
                continue
            r = dict(region_list(k, g[k]))[tag]
            p.grad = torch.tensor(g[k][r].copy())
            opts[(k, tag)].step()
    for (k, tag), p in params.items():
        r = dict(region_list(k, wt[k]))[tag]
        assert np.allclose(wt[k][r], p.detach().numpy(), rtol=1e-12, atol=1e-14), (k, tag)


def test_skipped_subnets_keep_weights_and_momentum_bitwise():
    w = tiny(heads=3, mlp=48)
    rng = np.random.default_rng(82)
    _, wt, _ = draw(w, 82)
    vt = {k: (None if a is None else rng.standard_normal(a.shape)) for k, a in wt.items()}
    g = {k: (None if a is None else rng.standard_normal(a.shape)) for k, a in wt.items()}
    w2, v2 = orc.sgd_momentum_step(wt, g, vt, [False, True, False], w.head_dim, 0.1, 0.9, 0.0, gate_ffn=True)
    for k, a in wt.items():
        if a is None or slices_of(k, a, 0, w, True) is None:
            continue
        for h in (0, 2):
            r = slices_of(k, a, h, w, True)
            assert np.array_equal(w2[k][r], np.asarray(a, np.float64)[r]) and np.array_equal(v2[k][r], vt[k][r]), k
        r = slices_of(k, a, 1, w, True)
        assert not np.array_equal(w2[k][r], np.asarray(a, np.float64)[r])
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
