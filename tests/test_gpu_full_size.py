"""GPU parity at the benchmark's full shapes and launch configuration (one block at a time).

The oracle computes a whole block in fp64 at full shape in seconds, so every element of every
output and gradient is compared (same bar as the small cases: 2e-2, bf16 storage).
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import TOL, compare_block, gpu_block, oracle_block, rel_inf

pytestmark = pytest.mark.gpu


def one_block(w, seed=0):
    """Block 0 of the workload's seeded draw: its input, weights, upstream gradient and op codes."""
    wb = di.scaled(w, blocks=1)
    rng = np.random.default_rng(seed)
    x = di.draw_hidden(rng, wb)
    wt = di.draw_block_weights(rng, wb)
    dy = di.draw_hidden(rng, wb)
    return wb, x, wt, dy


def check(w, ops, fields, seed=0):
    wb, x, wt, dy = one_block(w, seed)
    got = gpu_block(wb, wt, ops, x, dy, fields)
    ref = oracle_block(wb, wt, ops, x, dy)
    rep = {}
    compare_block(wb, ops, got, ref, TOL[w.dtype], fields, rep)
    print(f"[{w.name} full size ops={list(ops)}] " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()), flush=True)


BASE_FIELDS = tuple(k for k in di.WEIGHT_FIELDS if not k.startswith("ln") and not k.startswith("lora"))


def test_vit_b16_block_full_size():
    w = di.WORKLOADS["vit_b16"]
    ops = di.draw_stack(di.scaled(w, batch=1, blocks=w.blocks), 0).ops   # the benchmark's mask (cheap draw: batch 1)
    l = int(np.argmax([(o == di.OP_FWD).sum() + (o == di.OP_SKIP).sum() for o in ops]))   # the most mixed block
    check(w, list(ops[l]), BASE_FIELDS)


def test_vit_b16_block_full_size_all_full_and_no_full():
    w = di.WORKLOADS["vit_b16"]
    check(w, [di.OP_FULL] * w.heads, BASE_FIELDS, seed=1)
    check(w, [di.OP_FWD] * 6 + [di.OP_SKIP] * 6, BASE_FIELDS, seed=2)


def test_vit_l16_block_full_size():
    w = di.WORKLOADS["vit_l16"]
    ops = di.draw_stack(di.scaled(w, batch=1), 0).ops
    check(w, list(ops[3]), BASE_FIELDS)


def test_vit_b16_share_block_full_size_with_knapsack_codes():
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    w = di.WORKLOADS["vit_b16_share4"]
    ks = di.draw_stack(di.scaled(w, batch=1), 0).knapsack
    codes = P.d2ft_select_knapsack(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    ref = orc.knapsack_scheduling(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    assert np.array_equal(codes, ref)
    ops = codes.reshape(w.blocks, w.heads)
    l = int(np.argmax([len(set(o.tolist())) for o in ops]))
    check(w, list(ops[l]), BASE_FIELDS)


def test_vit_b16_lora_block_full_size():
    w = di.scaled(di.WORKLOADS["vit_b16_lora"], lora_b_zero=False)   # B != 0 so that dA is exercised
    ops = di.draw_stack(di.scaled(w, batch=1), 0).ops
    check(w, list(ops[0]), ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"))


def test_two_block_stack_full_size():
    import torch
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    w = di.scaled(di.WORKLOADS["vit_b16"], blocks=2)
    s = di.draw_stack(w, seed=3)
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype)
    dws = [{k: P.to_device(v, w.dtype) for k, v in bw.items()} for bw in s.weights]
    st = P.BlockStack(desc, dws, w.dtype)
    y, dx = st.step(P.to_device(s.x, w.dtype), P.to_device(s.dy, w.dtype), s.ops)
    torch.cuda.synchronize()
    ry, caches = orc.stack_fwd(s.weights, s.ops, s.x, w.head_dim)
    rdx, rgrads = orc.stack_bwd(s.weights, caches, s.dy)
    errs = {"y": rel_inf(y.float().cpu().numpy(), ry), "dx": rel_inf(dx.float().cpu().numpy(), rdx)}
    for l in range(w.blocks):
        for k in ("w_qkv", "w_o", "w1", "w2"):
            errs[f"d{k}[{l}]"] = rel_inf(st.grads[l][k].float().cpu().numpy(), rgrads[l][k])
    print("[two-block stack full size] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= 2e-2 for v in errs.values()), errs


@pytest.mark.parametrize("workload", ["vit_b16", "vit_b16_ffn"])
def test_micro_batched_block_full_size(workload):
    """The benchmark's --micro 5 configuration (13/13/13/13/12 images, one code per (subnet, micro-batch))."""
    from oracle import d2ft_oracle as orc
    from test_gpu_microbatch import gpu_block_mb
    from helpers import FLAG_GATE_FFN
    w = di.WORKLOADS[workload]
    wb, x, wt, dy = one_block(w, seed=5)
    mb = [13, 13, 13, 13, 12]
    ops_mb = di.exact_count_masks(np.random.default_rng(6), 5, w.heads, 0.6, 0.2, 0.2)
    assert all((o != di.OP_SKIP).any() for o in ops_mb)
    ops_mb = [list(o) for o in ops_mb]
    y, dx, g = gpu_block_mb(wb, wt, ops_mb, mb, x, dy, FLAG_GATE_FFN if w.gate_ffn else 0)
    ry, caches = orc.block_fwd_mb(wt, ops_mb, mb, x, w.head_dim, w.ln_eps, w.lora_scale, gate_ffn=w.gate_ffn)
    rdx, rg = orc.block_bwd_mb(wt, caches, mb, dy)
    errs = {"y": rel_inf(y, ry), "dx": rel_inf(dx, rdx)}
    for k in BASE_FIELDS:
        if g.get(k) is not None:
            errs["d" + k] = rel_inf(g[k], rg[k])
    print(f"[{w.name} full size, 5 micro-batches] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert all(v <= TOL[w.dtype] for v in errs.values()), errs
