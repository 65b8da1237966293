"""GPU parity at the benchmark's full shapes, launch configuration and op codes.

The oracle computes a whole block in fp64 at full shape in seconds, so every element of every
output and gradient is compared (same bar as the small cases: 2e-2, bf16 storage):
  * every block of the ViT-B/16 and ViT-L/16 stacks under the benchmark's own op codes, the oracle fed
    the GPU's own input and upstream gradient of that block (errors do not chain);
  * the same stacks end to end (errors chain over 12 / 24 bf16 blocks);
  * single blocks of the other workloads, and the micro-batched calls.
Gradients of per-head tensors are also checked slice by slice (one plane of one p_f head at a time),
so a wrong small-magnitude slice cannot hide behind the tensor's largest entry.
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import TOL, compare_block, gpu_block, oracle_block, rel_inf

pytestmark = pytest.mark.gpu


def per_head_slice_errors(w, ops, g, rg):
    """max |gpu - oracle| / max |oracle| over each (plane, p_f head) slice of w_qkv, b_qkv, w_o.
    The key plane of b_qkv is left out: that gradient is identically zero (softmax does not change when
    all keys of a head shift by a constant), so it is compared on the scale of the whole tensor instead."""
    dh, errs = w.head_dim, {}
    for h, o in enumerate(ops):
        if o != di.OP_FULL:
            continue
        for p in range(3):
            errs[f"dw_qkv[{p},{h}]"] = rel_inf(g["w_qkv"][p, h], rg["w_qkv"][p, h])
            if p != 1:
                errs[f"db_qkv[{p},{h}]"] = rel_inf(g["b_qkv"][p, h], rg["b_qkv"][p, h])
        errs[f"db_qkv[1,{h}]/all"] = float(np.abs(g["b_qkv"][1, h] - rg["b_qkv"][1, h]).max() / np.abs(rg["b_qkv"]).max())
        errs[f"dw_o[{h}]"] = rel_inf(g["w_o"][:, h * dh:(h + 1) * dh], rg["w_o"][:, h * dh:(h + 1) * dh])
    return errs


BASE_FIELDS = tuple(k for k in di.WEIGHT_FIELDS if not k.startswith("ln") and not k.startswith("lora"))

_runs = {}


def stack_run(name):
    """One step of the whole stack on the GPU as the benchmark runs it (same seed, same op codes, same
    launch sequence), keeping every block's input, output, upstream gradient, input gradient and weight
    gradients on the host."""
    if name in _runs:
        return _runs[name]
    _runs.clear()   # one workload's arrays at a time
    import torch
    import paper_2504_12471_amd as P
    w = di.WORKLOADS[name]
    s = di.draw_stack(w, 0)
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, P.FLAG_GATE_FFN if w.gate_ffn else 0)
    dws = [{k: P.to_device(v, w.dtype) for k, v in bw.items()} for bw in s.weights]
    st = P.BlockStack(desc, dws, w.dtype, BASE_FIELDS)
    for gl in st.grads:
        for t in gl.values():
            if t is not None:
                t.fill_(float("nan"))   # overwrite mode must replace every element
    host = lambda t: t.float().cpu().numpy()
    st.forward(P.to_device(s.x, w.dtype), s.ops)
    acts = [host(a) for a in st.acts]
    cur = P.to_device(s.dy, w.dtype)
    dys, dxs = [None] * w.blocks, [None] * w.blocks
    for l in range(w.blocks - 1, -1, -1):
        out = torch.empty_like(cur)
        P.d2ft_block_bwd(desc, dws[l], s.ops[l], st.acts[l], cur, out, st.grads[l], st.saved[l], st.scratch)
        dys[l], dxs[l] = host(cur), host(out)
        cur = out
    torch.cuda.synchronize()
    grads = [{k: (None if t is None else host(t)) for k, t in gl.items()} for gl in st.grads]
    _runs[name] = (w, s, acts, dys, dxs, grads)
    return _runs[name]


def check_block_of_stack(name, l):
    w, s, acts, dys, dxs, grads = stack_run(name)
    wb = di.scaled(w, blocks=1)
    ops = list(s.ops[l])
    ref = oracle_block(wb, s.weights[l], ops, acts[l], dys[l], gate_ffn=w.gate_ffn)
    rep = {}
    compare_block(wb, ops, (acts[l + 1], dxs[l], grads[l]), ref, TOL[w.dtype], BASE_FIELDS, rep, gate_ffn=w.gate_ffn)
    sl = per_head_slice_errors(wb, ops, grads[l], ref[2])
    worst = max(sl, key=sl.get) if sl else None
    print(f"[{name} block {l} ops={ops}] " + " ".join(f"{k}={v:.2e}" for k, v in rep.items())
          + (f" worst slice {worst}={sl[worst]:.2e}" if worst else ""), flush=True)
    bad = {k: v for k, v in sl.items() if not v <= TOL[w.dtype]}
    assert not bad, bad


def check_whole_stack(name):
    from oracle import d2ft_oracle as orc
    w, s, acts, dys, dxs, grads = stack_run(name)
    ry, caches = orc.stack_fwd(s.weights, s.ops, s.x, w.head_dim, w.ln_eps, w.lora_scale, gate_ffn=w.gate_ffn)
    rdx, rgrads = orc.stack_bwd(s.weights, caches, s.dy)
    errs = {"y": rel_inf(acts[-1], ry), "dx": rel_inf(dxs[0], rdx)}
    for l in range(w.blocks):
        for k in BASE_FIELDS:
            errs[f"d{k}[{l}]"] = rel_inf(grads[l][k], rgrads[l][k])
    worst = sorted(errs, key=errs.get)[-3:]
    # The hidden state is rounded to the storage type twice per block and those roundings are independent,
    # so over a chain of L blocks they add in quadrature: the bar of one step through 12 blocks (2e-2) is
    # scaled by sqrt(L / 12) for deeper stacks.  Every block on its own is held to 2e-2 above.
    tol = TOL[w.dtype] * max(1.0, (w.blocks / 12.0) ** 0.5)
    print(f"[{name} whole stack, {w.blocks} blocks, bar {tol:.2e}] y={errs['y']:.2e} dx={errs['dx']:.2e} worst: "
          + " ".join(f"{k}={errs[k]:.2e}" for k in worst), flush=True)
    assert all(v <= tol for v in errs.values()), {k: v for k, v in errs.items() if not v <= tol}


@pytest.mark.parametrize("l", range(12))
def test_vit_b16_every_block_full_size(l):
    check_block_of_stack("vit_b16", l)


def test_vit_b16_whole_stack_full_size():
    check_whole_stack("vit_b16")


@pytest.mark.parametrize("l", range(24))
def test_vit_l16_every_block_full_size(l):
    check_block_of_stack("vit_l16", l)


def test_vit_l16_whole_stack_full_size():
    check_whole_stack("vit_l16")


@pytest.mark.parametrize("l", [0, 4, 8])
def test_vit_b16_ffn_blocks_full_size(l):
    check_block_of_stack("vit_b16_ffn", l)


def test_release_stack_arrays():
    _runs.clear()


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


def test_vit_b16_block_full_size_all_full_and_no_full():
    w = di.WORKLOADS["vit_b16"]
    check(w, [di.OP_FULL] * w.heads, BASE_FIELDS, seed=1)
    check(w, [di.OP_FWD] * 6 + [di.OP_SKIP] * 6, BASE_FIELDS, seed=2)


def test_vit_b16_share_block_full_size_with_knapsack_codes():
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    w = di.WORKLOADS["vit_b16_share4"]
    ks = di.draw_ops(w, 0)[1]
    codes = P.d2ft_select_knapsack(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    ref = orc.knapsack_scheduling(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    assert np.array_equal(codes, ref)
    ops = codes.reshape(w.blocks, w.heads)
    l = int(np.argmax([len(set(o.tolist())) for o in ops]))
    check(w, list(ops[l]), BASE_FIELDS)


def test_vit_b16_lora_block_full_size():
    w = di.scaled(di.WORKLOADS["vit_b16_lora"], lora_b_zero=False)   # B != 0 so that dA is exercised
    ops = di.draw_ops(w, 0)[0]
    check(w, list(ops[0]), ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"))


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
