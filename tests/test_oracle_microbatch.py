"""Pins for the oracle's micro-batched block (one op code per (subnet, micro-batch), Alg. 1 T_opt[k][x_i]).  No GPU.

  * equal codes in every micro-batch == one call over the whole batch (images are independent in a block),
  * torch fp64 autograd of the sum of the micro-batches' objectives with per-micro-batch detach patterns:
    shared parameters collect the summed gradient,
  * a subnet that is p_f in no micro-batch gets exact zeros; in one micro-batch, exactly that one's gradient.
"""
import numpy as np
import pytest
import torch

import d2ft_inputs as di
from oracle import d2ft_oracle as orc
from test_oracle_block import draw, relerr, tiny, torch_block
from test_oracle_ffn_gate import torch_gated_block

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def test_equal_codes_equal_the_whole_batch_call():
    w = tiny(heads=3, batch=5)
    x, wt, dy = draw(w, 61)
    ops = [FULL, FWD, SKIP]
    y, caches = orc.block_fwd_mb(wt, [ops, ops, ops], [2, 1, 2], x, w.head_dim)
    dx, g = orc.block_bwd_mb(wt, caches, [2, 1, 2], dy)
    y0, c0 = orc.block_fwd(wt, ops, x, w.head_dim)
    dx0, g0 = orc.block_bwd(wt, c0, dy)
    assert relerr(y, y0) < 1e-13 and relerr(dx, dx0) < 1e-12
    for k in g0:
        if g0[k] is not None:
            assert relerr(g[k], g0[k]) < 1e-12, k


@pytest.mark.parametrize("gate", [False, True])
def test_micro_batches_match_autograd_of_the_summed_objective(gate):
    w = tiny(heads=3, batch=6, mlp=48)
    x, wt, dy = draw(w, 62)
    ops_mb = [[FULL, FWD, SKIP], [SKIP, FULL, FULL], [FWD, FWD, SKIP]]
    mb = [1, 3, 2]
    y, caches = orc.block_fwd_mb(wt, ops_mb, mb, x, w.head_dim, gate_ffn=gate)
    dx, g = orc.block_bwd_mb(wt, caches, mb, dy)
    # torch: one set of leaf parameters, one graph per micro-batch, gradients accumulate in .grad
    P = {k: (None if v is None else torch.tensor(np.asarray(v, np.float64), requires_grad=True)) for k, v in wt.items()}
    b0, ys, dxs = 0, [], []
    build = torch_gated_block if gate else torch_block
    for ops, nb in zip(ops_mb, mb):
        ref, xt, Pi = build(wt, ops, x[b0:b0 + nb], w.head_dim)
        ref.backward(torch.tensor(dy[b0:b0 + nb]))
        ys.append(ref.detach().numpy()); dxs.append(xt.grad.numpy())
        for k, p in Pi.items():
            if p is not None and p.grad is not None:
                P[k].grad = p.grad.clone() if P[k].grad is None else P[k].grad + p.grad
        b0 += nb
    assert relerr(y, np.concatenate(ys)) < 1e-12
    assert relerr(dx, np.concatenate(dxs)) < 1e-11
    for k, p in P.items():
        if p is None:
            continue
        gr = np.zeros(p.shape) if p.grad is None else p.grad.numpy()
        if np.abs(gr).max() == 0.0:
            assert np.all(g[k] == 0.0), k
        else:
            assert relerr(g[k], gr) < 1e-10, k


def test_subnet_gradients_come_only_from_micro_batches_where_it_is_full():
    w = tiny(heads=2, batch=4)
    x, wt, dy = draw(w, 63)
    ops_mb = [[FULL, SKIP], [FWD, SKIP], [SKIP, FWD]]
    mb = [2, 1, 1]
    _, caches = orc.block_fwd_mb(wt, ops_mb, mb, x, w.head_dim)
    _, g = orc.block_bwd_mb(wt, caches, mb, dy)
    _, c0 = orc.block_fwd(wt, ops_mb[0], x[:2], w.head_dim)
    _, g0 = orc.block_bwd(wt, c0, dy[:2])
    dh = w.head_dim
    assert np.array_equal(g["w_qkv"][:, 0], g0["w_qkv"][:, 0])            # head 0: micro-batch 0 alone
    assert np.array_equal(g["w_o"][:, :dh], g0["w_o"][:, :dh])
    assert np.all(g["w_qkv"][:, 1] == 0.0) and np.all(g["w_o"][:, dh:] == 0.0) and np.all(g["b_qkv"][:, 1] == 0.0)
