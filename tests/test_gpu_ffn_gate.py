"""GPU parity for D2FT_FLAG_GATE_FFN: the op code of head h also governs hidden units
[h*Dm/H, (h+1)*Dm/H) of the feed-forward network (the subnet of Sec. II-A.1), against the oracle's
gate_ffn path.  Same bar as the other block tests; the feed-forward gradient slices of subnets that
are not p_f must be exactly +0.0.
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import FLAG_GATE_FFN, TOL, compare_block, gpu_block, oracle_block, rel_inf

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def draw_block(w, seed):
    rng = np.random.default_rng(seed)
    x = di.draw_hidden(rng, w)
    wt = di.draw_block_weights(rng, w)
    dy = di.draw_hidden(rng, w)
    return x, wt, dy


def run_gated(w, ops, seed=0, flags=0, grad_fields=None):
    x, wt, dy = draw_block(w, seed)
    fields = di.WEIGHT_FIELDS if grad_fields is None else grad_fields
    got = gpu_block(w, wt, ops, x, dy, fields, flags | FLAG_GATE_FFN)
    ref = oracle_block(w, wt, ops, x, dy, gate_ffn=True)
    rep = {}
    compare_block(w, ops, got, ref, TOL[w.dtype], fields, rep, gate_ffn=True)
    print(f"[gated {w.name} ops={list(ops)} flags={flags}] " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()), flush=True)
    return got, ref, (x, wt, dy)


@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP), (FULL, FULL, FULL), (SKIP, SKIP, SKIP), (FWD, FWD, FWD),
                                 (SKIP, FULL, SKIP), (FWD, SKIP, SKIP), (SKIP, FWD, FULL)])
def test_fp32_gated_masks(ops):
    run_gated(di.WORKLOADS["vit_tiny_fp32"], list(ops), seed=31)


def test_fp32_gated_all_shortcut_is_the_identity_bitwise():
    w = di.WORKLOADS["vit_tiny_fp32"]
    (y, dx, g), _, (x, wt, dy) = run_gated(w, [SKIP] * 3, seed=32)
    assert np.array_equal(y, x.reshape(y.shape).astype(np.float32))
    assert np.array_equal(dx, dy.reshape(dx.shape).astype(np.float32))
    for k, v in g.items():
        if v is not None:
            assert np.all(v == 0.0) and not np.any(np.signbit(v)), k


def test_fp32_gated_all_full_equals_ungated_run():
    w = di.WORKLOADS["vit_tiny_fp32"]
    x, wt, dy = draw_block(w, 33)
    a = gpu_block(w, wt, [FULL] * 3, x, dy, di.WEIGHT_FIELDS, FLAG_GATE_FFN)
    b = gpu_block(w, wt, [FULL] * 3, x, dy, di.WEIGHT_FIELDS, 0)
    assert rel_inf(a[0], b[0]) < 1e-6 and rel_inf(a[1], b[1]) < 1e-6
    for k in a[2]:
        if a[2][k] is not None:
            assert rel_inf(a[2][k], b[2][k]) < 1e-5, k


def test_gated_accumulate_mode_leaves_non_full_slices():
    w = di.WORKLOADS["vit_tiny_fp32"]
    x, wt, dy = draw_block(w, 34)
    ops = [FULL, FWD, SKIP]
    rng = np.random.default_rng(35)
    init = {k: (rng.standard_normal(v.shape) * 0.1).astype(np.float32) for k, v in wt.items() if v is not None}
    _, _, g = gpu_block(w, wt, ops, x, dy, di.WEIGHT_FIELDS, flags=1 | FLAG_GATE_FFN, grads_init=init)
    _, _, rg, _ = oracle_block(w, wt, ops, x, dy, gate_ffn=True)
    for k, v in g.items():
        if v is not None:
            assert rel_inf(v, init[k] + rg[k]) < 1e-4, k
    S = w.mlp_hidden // w.heads
    for h in (1, 2):   # not p_f: untouched, bit for bit
        assert np.array_equal(g["w1"][h * S:(h + 1) * S], init["w1"][h * S:(h + 1) * S])
        assert np.array_equal(g["b1"][h * S:(h + 1) * S], init["b1"][h * S:(h + 1) * S])
        assert np.array_equal(g["w2"][:, h * S:(h + 1) * S], init["w2"][:, h * S:(h + 1) * S])


def test_gate_needs_slices_of_whole_64_column_blocks():
    import torch
    import paper_2504_12471_amd as P
    w = di.Workload("bad_slice", 1, 8, 64, 3, 64, 480, 1, "f32")   # 480 / 3 = 160, not a multiple of 64
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, 0, 1.0, w.ln_eps, w.head_dim,
                       FLAG_GATE_FFN)
    assert P.d2ft_block_saved_bytes(desc) == 0 and P.d2ft_block_scratch_bytes(desc) == 0


SMALL_BF16 = di.Workload("small_bf16_gate", 3, 70, 256, 4, 64, 512, 1, "bf16")       # slices of 128 hidden units
MID_BF16 = di.Workload("mid_bf16_gate", 5, 197, 384, 6, 64, 1536, 1, "bf16")       # ViT-Small block, slices of 256


@pytest.mark.parametrize("flags", [0, 2])
@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP, FULL), (FULL,) * 4, (SKIP,) * 4, (FWD, FWD, SKIP, FWD)])
def test_bf16_gated_small(ops, flags):
    run_gated(SMALL_BF16, list(ops), seed=36, flags=flags)


@pytest.mark.parametrize("flags", [0, 2])
def test_bf16_gated_vit_small_block(flags):
    run_gated(MID_BF16, [FULL, SKIP, FWD, FULL, FULL, SKIP], seed=37, flags=flags)


def test_bf16_gated_frozen_fields_and_null_biases():
    x, wt, dy = draw_block(SMALL_BF16, 38)
    wt["b_o"] = None
    wt["b2"] = None
    fields = ("w_qkv", "w1", "b1")
    ops = [FWD, FULL, SKIP, FULL]
    got = gpu_block(SMALL_BF16, wt, ops, x, dy, fields, FLAG_GATE_FFN)
    ref = oracle_block(SMALL_BF16, wt, ops, x, dy, gate_ffn=True)
    compare_block(SMALL_BF16, ops, got, ref, TOL["bf16"], fields, gate_ffn=True)
    assert got[2]["w2"] is None and got[2]["b2"] is None


def test_bf16_gated_full_size_vit_b16_block():
    """One ViT-B/16 block at the benchmark's shape with the gated mask of block 0."""
    w = di.WORKLOADS["vit_b16"]
    s = di.draw_stack(w, 0)
    ops = list(s.ops[0])
    rng = np.random.default_rng(39)
    x, dy = di.draw_hidden(rng, w), di.draw_hidden(rng, w)
    got = gpu_block(w, s.weights[0], ops, x, dy, di.WEIGHT_FIELDS, FLAG_GATE_FFN)
    ref = oracle_block(w, s.weights[0], ops, x, dy, gate_ffn=True)
    rep = {}
    compare_block(w, ops, got, ref, TOL["bf16"], di.WEIGHT_FIELDS, rep, gate_ffn=True)
    print("[gated vit_b16 block 0 ops=%s] " % ops + " ".join(f"{k}={v:.2e}" for k, v in rep.items()), flush=True)
