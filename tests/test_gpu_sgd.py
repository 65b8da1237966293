"""GPU parity for d2ft_sgd_step (SGD with momentum on the slices of the p_f subnets, Sec. IV-A) against the oracle.

fp32 arithmetic on the GPU against fp64 on the CPU: 1e-6 relative for fp32 tensors and fp32 master copies,
2^-8 relative for bf16 weights without a master copy (one rounding to storage).  Slices of subnets that are
not p_f must stay bit for bit, momentum and master copy included.
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import FLAG_GATE_FFN, rel_inf

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def run_sgd(w, ops, seed, gate, use_master, steps=2, frozen=()):
    import torch
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    rng = np.random.default_rng(seed)
    flags = FLAG_GATE_FFN if gate else 0
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, flags)
    wt = di.draw_block_weights(rng, w)
    wt = {k: (None if a is None else a * 20.0) for k, a in wt.items()}
    if w.dtype == "bf16":
        wt = {k: (None if a is None else di.round_to_bf16(a)) for k, a in wt.items()}
    dev_w = {k: P.to_device(a, w.dtype) for k, a in wt.items()}
    dev_v = {k: (None if a is None else torch.zeros(a.shape, dtype=torch.float32, device="cuda")) for k, a in wt.items()}
    dev_m = ({k: (None if a is None else torch.tensor(a, dtype=torch.float32, device="cuda")) for k, a in wt.items()}
             if use_master else None)
    ref_w = {k: (None if a is None else np.asarray(a, np.float64)) for k, a in wt.items()}
    ref_v = {k: (None if a is None else np.zeros(a.shape)) for k, a in wt.items()}
    lr, mu, wd = 0.05, 0.9, 0.01
    updated = [o == FULL for o in ops]
    for _ in range(steps):
        g = {k: (None if (a is None or k in frozen) else rng.standard_normal(a.shape).astype(np.float32))
             for k, a in wt.items()}
        if w.dtype == "bf16":
            g = {k: (None if a is None else di.round_to_bf16(a)) for k, a in g.items()}
        dev_g = {k: P.to_device(a, w.dtype) for k, a in g.items()}
        before = {k: (None if t is None else t.clone()) for k, t in dev_w.items()}
        P.d2ft_sgd_step(desc, dev_w, dev_g, dev_v, dev_m, ops, lr, mu, wd)
        torch.cuda.synchronize()
        new_w, new_v = orc.sgd_momentum_step(ref_w, g, ref_v, updated, w.head_dim, lr, mu, wd, gate_ffn=gate)
        tol_w = 1e-6 if (w.dtype == "f32" or use_master) else 2.0 ** -8
        for k, a in new_w.items():
            if a is None:
                continue
            got = (dev_m[k] if use_master else dev_w[k]).double().cpu().numpy()
            assert rel_inf(got, a) <= tol_w, (k, rel_inf(got, a))
            assert rel_inf(dev_v[k].double().cpu().numpy(), new_v[k]) <= 1e-6 or np.abs(new_v[k]).max() == 0.0, k
            if use_master and w.dtype == "bf16":   # the storage copy is the rounded master copy
                assert torch.equal(dev_w[k], dev_m[k].to(torch.bfloat16)), k
            # slices of subnets that are not p_f: bit for bit
            for h, up in enumerate(updated):
                r = orc._head_slices(k, a, h, w.heads, w.head_dim, gate)
                if r is not None and not up:
                    assert torch.equal(dev_w[k][r], before[k][r]), (k, h)
                    assert float(dev_v[k][r].abs().max()) == 0.0, (k, h)
            if g[k] is None:
                assert torch.equal(dev_w[k], before[k]), k
        # carry on from the GPU state (rounded weights), keeping the two sides on the same inputs
        ref_w = {k: (None if t is None else (dev_m[k] if use_master else t).double().cpu().numpy()) for k, t in dev_w.items()}
        ref_v = {k: (None if t is None else t.double().cpu().numpy()) for k, t in dev_v.items()}


@pytest.mark.parametrize("gate", [False, True])
def test_fp32_sgd(gate):
    run_sgd(di.WORKLOADS["vit_tiny_fp32"], [FULL, FWD, SKIP], 91, gate, use_master=False)


@pytest.mark.parametrize("use_master", [False, True])
@pytest.mark.parametrize("gate", [False, True])
def test_bf16_lora_sgd(gate, use_master):
    w = di.Workload("sgd_lora", 2, 33, 128, 4, 64, 256, 1, "bf16", lora_rank=8, lora_b_zero=False)
    run_sgd(w, [FULL, SKIP, FWD, FULL], 92, gate, use_master)


def test_no_full_subnet_updates_shared_tensors_only():
    run_sgd(di.WORKLOADS["vit_tiny_fp32"], [FWD, SKIP, SKIP], 93, True, use_master=False)


def test_frozen_fields_are_untouched():
    run_sgd(di.WORKLOADS["vit_tiny_fp32"], [FULL, FULL, SKIP], 94, False, use_master=False,
            frozen=("ln1_g", "ln1_b", "ln2_g", "ln2_b", "w_o"))


def test_full_size_block_sgd():
    run_sgd(di.scaled(di.WORKLOADS["vit_b16_ffn"], batch=1), [FULL] * 6 + [SKIP, FWD, SKIP, SKIP, FULL, SKIP], 95, True,
            use_master=True, steps=1)
