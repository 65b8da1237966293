"""GPU parity for d2ft_subnet_scores (Sec. II-B contribution scores) against the oracle.

The kernels accumulate in fp64 over inputs that are exactly representable, so the bar is 1e-12
relative per score (summation order is the only difference from the oracle).
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import FLAG_GATE_FFN, gpu_block

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def gpu_scores(w, tensors, kind, flags=0):
    import paper_2504_12471_amd as P
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, flags)
    dev = {k: P.to_device(v, w.dtype) for k, v in tensors.items()}
    return P.d2ft_subnet_scores(desc, dev, kind)


def check(w, tensors, gate):
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    flags = FLAG_GATE_FFN if gate else 0
    for kind, name in ((P.SCORE_FISHER, "fisher"), (P.SCORE_MAGNITUDE, "magnitude")):
        got = gpu_scores(w, tensors, kind, flags)
        ref = orc.subnet_scores(tensors, w.heads, w.head_dim, name, gate_ffn=gate)
        err = np.abs(got - ref).max() / np.abs(ref).max()
        print(f"[scores {w.name} {name} gate={gate}] max rel err {err:.2e}", flush=True)
        assert np.all(np.abs(got - ref) <= 1e-12 * np.abs(ref).max())


@pytest.mark.parametrize("gate", [False, True])
def test_fp32_weight_scores(gate):
    w = di.WORKLOADS["vit_tiny_fp32"]
    wt = di.draw_block_weights(np.random.default_rng(51), w)
    check(w, wt, gate)


@pytest.mark.parametrize("gate", [False, True])
def test_bf16_lora_weight_scores(gate):
    w = di.Workload("scores_lora", 2, 33, 128, 4, 64, 256, 1, "bf16", lora_rank=8, lora_b_zero=False)
    wt = di.draw_block_weights(np.random.default_rng(52), w)
    check(w, wt, gate)


def test_null_fields_are_skipped():
    w = di.WORKLOADS["vit_tiny_fp32"]
    wt = di.draw_block_weights(np.random.default_rng(53), w)
    wt = {k: (v if k in ("w_qkv", "w2", "b1") else None) for k, v in wt.items()}
    check(w, wt, True)


def test_fisher_scores_of_gpu_gradients_full_size_block():
    """Gradients of one ViT-B/16 block computed on the GPU, scored on the GPU and by the oracle from the same arrays."""
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    w = di.WORKLOADS["vit_b16_ffn"]
    s = di.draw_stack(w, 0)
    rng = np.random.default_rng(54)
    x, dy = di.draw_hidden(rng, w), di.draw_hidden(rng, w)
    ops = [FULL] * w.heads   # scores are collected with every subnet trained (before fine-tuning, Sec. II-B)
    _, _, g = gpu_block(w, s.weights[0], ops, x, dy, di.WEIGHT_FIELDS, FLAG_GATE_FFN)
    got = gpu_scores(w, g, P.SCORE_FISHER, FLAG_GATE_FFN)
    ref = orc.subnet_scores(g, w.heads, w.head_dim, "fisher", gate_ffn=True)
    assert np.all(np.abs(got - ref) <= 1e-12 * np.abs(ref).max())
    assert np.all(got > 0)


def test_scores_reject_bad_arguments():
    import torch
    import paper_2504_12471_amd as P
    w = di.WORKLOADS["vit_tiny_fp32"]
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype)
    dev = {k: P.to_device(v, w.dtype) for k, v in di.draw_block_weights(np.random.default_rng(55), w).items()}
    with pytest.raises(P.D2ftError):
        P.d2ft_subnet_scores(desc, dev, 7)
    with pytest.raises(P.D2ftError):
        P.d2ft_subnet_scores(desc, dev, P.SCORE_FISHER, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
