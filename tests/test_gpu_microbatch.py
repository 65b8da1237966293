"""GPU parity for d2ft_block_fwd_mb / d2ft_block_bwd_mb: one op code per (subnet, micro-batch)
(Alg. 1, T_opt[k][x_i]), weight gradients added over the micro-batches, against the oracle."""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import FLAG_GATE_FFN, TOL, rel_inf

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def gpu_block_mb(w, weights, ops_mb, mb, x, dy, flags=0, grads_init=None):
    import torch
    import paper_2504_12471_amd as P
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, w.lora_rank, w.lora_scale,
                       w.ln_eps, w.head_dim, flags)
    dw = {k: P.to_device(v, w.dtype) for k, v in weights.items()}
    xd, dyd = P.to_device(x, w.dtype), P.to_device(dy, w.dtype)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    saved = torch.empty(P.d2ft_block_saved_bytes_mb(desc, mb), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(P.d2ft_block_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    grads = {k: (None if v is None else (torch.full_like(v, float("nan")) if grads_init is None
                                         else P.to_device(grads_init[k], w.dtype))) for k, v in dw.items()}
    P.d2ft_block_fwd_mb(desc, dw, mb, ops_mb, xd, y, saved, scratch)
    P.d2ft_block_bwd_mb(desc, dw, mb, ops_mb, xd, dyd, dx, grads, saved, scratch)
    torch.cuda.synchronize()
    host = lambda t: None if t is None else t.float().cpu().numpy()
    return host(y), host(dx), {k: host(v) for k, v in grads.items()}


def run_mb(w, ops_mb, mb, seed, gate=False):
    from oracle import d2ft_oracle as orc
    rng = np.random.default_rng(seed)
    x, wt, dy = di.draw_hidden(rng, w), di.draw_block_weights(rng, w), di.draw_hidden(rng, w)
    y, dx, g = gpu_block_mb(w, wt, ops_mb, mb, x, dy, FLAG_GATE_FFN if gate else 0)
    ry, caches = orc.block_fwd_mb(wt, ops_mb, mb, x, w.head_dim, w.ln_eps, w.lora_scale, gate_ffn=gate)
    rdx, rg = orc.block_bwd_mb(wt, caches, mb, dy)
    tol = TOL[w.dtype]
    errs = {"y": rel_inf(y, ry), "dx": rel_inf(dx, rdx)}
    for k, v in g.items():
        if v is not None:
            assert np.all(np.isfinite(v)), k
            errs["d" + k] = rel_inf(v, rg[k])
    print(f"[mb {w.name} mb={mb} gate={gate}] " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    # a subnet that is p_f in no micro-batch: exact +0.0
    dh = w.head_dim
    for h in range(w.heads):
        if all(ops[h] != FULL for ops in ops_mb):
            for s in (g["w_qkv"][:, h], g["b_qkv"][:, h], g["w_o"][:, h * dh:(h + 1) * dh]):
                assert np.all(s == 0.0) and not np.any(np.signbit(s))
    return g, rg


def test_fp32_three_micro_batches():
    w = di.scaled(di.WORKLOADS["vit_tiny_fp32"], batch=6)
    run_mb(w, [[FULL, FWD, SKIP], [SKIP, FULL, SKIP], [FWD, FWD, SKIP]], [1, 3, 2], seed=71)


def test_fp32_micro_batches_without_a_live_or_full_subnet():
    """First micro-batch all-shortcut (x1 = x, b_o not applied), second forward-only, third mixed."""
    w = di.scaled(di.WORKLOADS["vit_tiny_fp32"], batch=6)
    run_mb(w, [[SKIP, SKIP, SKIP], [FWD, SKIP, FWD], [FULL, FWD, SKIP]], [2, 1, 3], seed=77)
    run_mb(w, [[FWD, FWD, FWD], [SKIP, SKIP, SKIP]], [4, 2], seed=78)      # nothing is p_f anywhere


def test_fp32_gated_micro_batches():
    w = di.scaled(di.WORKLOADS["vit_tiny_fp32"], batch=5)
    run_mb(w, [[FULL, SKIP, SKIP], [SKIP, SKIP, SKIP], [FWD, FULL, SKIP]], [2, 1, 2], seed=72, gate=True)


def test_single_micro_batch_equals_plain_call_bitwise():
    from helpers import gpu_block
    w = di.WORKLOADS["vit_tiny_fp32"]
    rng = np.random.default_rng(73)
    x, wt, dy = di.draw_hidden(rng, w), di.draw_block_weights(rng, w), di.draw_hidden(rng, w)
    ops = [FULL, FWD, SKIP]
    a = gpu_block_mb(w, wt, [ops], [w.batch], x, dy)
    b = gpu_block(w, wt, ops, x, dy)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for k in a[2]:
        if a[2][k] is not None:
            assert np.array_equal(a[2][k], b[2][k]), k


def test_bf16_five_micro_batches():
    w = di.Workload("mb_bf16", 10, 197, 384, 6, 64, 1536, 1, "bf16")
    rng = np.random.default_rng(74)
    ops_mb = [list(rng.choice([FULL, FULL, FULL, FWD, SKIP], size=w.heads)) for _ in range(5)]
    run_mb(w, ops_mb, [2, 2, 2, 2, 2], seed=75)
    run_mb(w, ops_mb, [3, 1, 2, 2, 2], seed=76, gate=True)


# bf16 with several micro-batches, each with a live head: the block runs once under the union of the codes
# and the attention kernels take the micro-batches' own codes as a mask.
def test_bf16_union_of_codes_mixed():
    w = di.Workload("mb_union", 7, 197, 384, 6, 64, 1536, 1, "bf16")
    ops_mb = [[FULL, FWD, SKIP, FULL, FWD, SKIP],
              [FWD, FWD, FWD, SKIP, SKIP, SKIP],       # nothing p_f in this micro-batch
              [SKIP, FULL, FULL, FWD, SKIP, SKIP]]     # head 1: forward-only, forward-only, p_f; head 5 never live
    g, rg = run_mb(w, ops_mb, [3, 1, 3], seed=81)
    assert np.all(g["w_qkv"][:, 5] == 0.0) and np.all(g["w_qkv"][:, 4] == 0.0)     # never p_f


def test_bf16_union_of_codes_gated_feed_forward():
    w = di.Workload("mb_union_gate", 6, 100, 384, 6, 64, 1536, 1, "bf16")
    ops_mb = [[FULL, FWD, SKIP, FULL, FWD, SKIP],
              [FWD, SKIP, FWD, SKIP, SKIP, SKIP],
              [SKIP, FULL, FULL, FWD, SKIP, SKIP]]
    g, rg = run_mb(w, ops_mb, [2, 1, 3], seed=86, gate=True)
    S = w.mlp_hidden // w.heads
    for h in (4, 5):   # never p_f: exact zeros in the slice's gradients
        assert np.all(g["w1"][h * S:(h + 1) * S] == 0.0) and np.all(g["w2"][:, h * S:(h + 1) * S] == 0.0)


def segment_launches(fn):
    """Runs fn with the library's per-kernel timing on; returns the launches of the row-segment GEMM kernels."""
    import paper_2504_12471_amd as P
    P.d2ft_timing_enable(True)
    try:
        fn()
        recs = P.d2ft_timing_read(256)
    finally:
        P.d2ft_timing_enable(False)
    # the kernel's template arguments end with (grouped, row segments, dz epilogue)
    return sum(r["launches"] for r in recs
               if r["name"].startswith("gemm_mfma_kernel<") and r["name"].rstrip(">").split(", ")[-2] == "true")


def test_bf16_gated_segments_slices_across_tiles_and_ends_inside_tiles():
    """Gated feed-forward products over row segments: slices of 192 columns (positions straddle the 256-column
    tiles), micro-batch ends inside the 256-row tiles, tiles without work (only head 0 lives in the last micro-
    batch, nothing is p_f in the second), a single-image micro-batch."""
    w = di.Workload("mb_seg_192", 9, 70, 512, 8, 64, 1536, 1, "bf16")
    ops_mb = [[FULL, FWD, SKIP, FULL, FWD, SKIP, FULL, SKIP],
              [FWD, SKIP, FWD, SKIP, SKIP, FWD, SKIP, SKIP],
              [SKIP, FULL, FULL, FWD, SKIP, SKIP, FULL, FWD],
              [FULL, SKIP, SKIP, SKIP, SKIP, SKIP, SKIP, SKIP]]
    n = segment_launches(lambda: run_mb(w, ops_mb, [1, 3, 2, 3], seed=91, gate=True))
    assert n == 2   # FC1 forward and the backward's dz


def test_bf16_gated_segments_eight_micro_batches_and_the_fallback_beyond():
    """Slices of 128 columns (two positions per tile column) over 8 micro-batches, the most the segment form
    takes; with 9 the same block runs the union of the slices over all rows and zeroes afterwards."""
    w = di.Workload("mb_seg_128", 12, 50, 256, 12, 64, 1536, 1, "bf16")
    rng = np.random.default_rng(92)
    ops8 = [list(rng.choice([FULL, FULL, FWD, SKIP, SKIP], size=w.heads)) for _ in range(8)]
    for o in ops8:
        o[0] = FULL
    n = segment_launches(lambda: run_mb(w, ops8, [2, 1, 2, 1, 2, 1, 2, 1], seed=92, gate=True))
    assert n == 2
    ops9 = ops8 + [ops8[0]]
    n = segment_launches(lambda: run_mb(w, ops9, [2, 1, 2, 1, 2, 1, 1, 1, 1], seed=93, gate=True))
    assert n == 0


def k_segment_launches(fn):
    """Runs fn with the library's per-kernel timing on; returns the launches of the GEMMs whose K walk follows the
    micro-batches' own slices (FC2 forward and the backward's dv)."""
    import paper_2504_12471_amd as P
    P.d2ft_timing_enable(True)
    try:
        fn()
        recs = P.d2ft_timing_read(256)
    finally:
        P.d2ft_timing_enable(False)
    return sum(r["launches"] for r in recs if r["name"].endswith("k-segments"))


def test_bf16_gated_k_walk_per_micro_batch():
    """FC2 forward and dv (and the output projection and du over the heads) walk, per tile, only the slices of the
    tile's own micro-batch: micro-batches that start at
    odd rows, a micro-batch smaller than a tile, one in which nothing is p_f (dv's tiles there walk nothing) and
    one with a single live subnet; then nine micro-batches, one more than the form takes (the full walk runs)."""
    w = di.Workload("mb_kseg", 9, 197, 384, 6, 64, 1536, 1, "bf16")
    ops_mb = [[FULL, FWD, SKIP, FULL, FWD, SKIP],
              [FWD, SKIP, FWD, SKIP, SKIP, FWD],
              [SKIP, FULL, FULL, FWD, SKIP, SKIP],
              [SKIP, SKIP, SKIP, SKIP, SKIP, FULL],
              [FULL, FULL, FULL, FULL, FULL, FULL]]
    n = k_segment_launches(lambda: run_mb(w, ops_mb, [3, 1, 2, 1, 2], seed=94, gate=True))
    assert n == 4   # with the output projection and du, whose K index runs over the heads
    n = k_segment_launches(lambda: run_mb(w, ops_mb, [3, 1, 2, 1, 2], seed=96))
    assert n == 2   # no gated slices: those two alone
    ops9 = ops_mb + [ops_mb[0], ops_mb[2], ops_mb[4], ops_mb[1]]
    n = k_segment_launches(lambda: run_mb(w, ops9, [1, 1, 1, 1, 1, 1, 1, 1, 1], seed=95, gate=True))
    assert n == 0


def test_bf16_union_of_codes_without_a_full_head():
    w = di.Workload("mb_union_fwd", 4, 100, 256, 4, 64, 512, 1, "bf16")
    g, rg = run_mb(w, [[FWD, SKIP, SKIP, FWD], [SKIP, FWD, SKIP, SKIP]], [1, 3], seed=82)
    for k in ("w_qkv", "b_qkv", "w_o"):
        assert np.all(g[k] == 0.0), k


def test_bf16_union_of_codes_ragged_tokens_and_single_images():
    w = di.Workload("mb_union_ragged", 5, 33, 128, 2, 64, 256, 1, "bf16")
    run_mb(w, [[FULL, SKIP], [SKIP, FULL], [FWD, FULL], [FULL, FULL], [FULL, FWD]], [1, 1, 1, 1, 1], seed=83)


def test_bf16_union_of_codes_with_lora():
    w = di.Workload("mb_union_lora", 6, 64, 256, 4, 64, 512, 1, "bf16", lora_rank=8, lora_scale=2.0, lora_b_zero=False)
    run_mb(w, [[FULL, FWD, SKIP, FULL], [SKIP, FULL, FULL, FWD]], [2, 4], seed=84)


def test_bf16_union_accumulates_into_existing_gradients():
    from oracle import d2ft_oracle as orc
    w = di.Workload("mb_union_acc", 4, 64, 128, 2, 64, 256, 1, "bf16")
    rng = np.random.default_rng(85)
    x, wt, dy = di.draw_hidden(rng, w), di.draw_block_weights(rng, w), di.draw_hidden(rng, w)
    ops_mb, mb = [[FULL, SKIP], [FWD, FULL]], [2, 2]
    init = {k: (None if v is None else np.asarray(rng.standard_normal(v.shape), np.float32)) for k, v in wt.items()}
    _, _, g = gpu_block_mb(w, wt, ops_mb, mb, x, dy, 1, grads_init=init)   # D2FT_FLAG_ACCUM_GRADS
    _, caches = orc.block_fwd_mb(wt, ops_mb, mb, x, w.head_dim, w.ln_eps, w.lora_scale)
    _, rg = orc.block_bwd_mb(wt, caches, mb, dy)
    for k, v in g.items():
        if v is not None:
            ref = np.asarray(init[k], np.float64) + rg[k]
            assert rel_inf(v, ref) <= 2 * TOL[w.dtype], k


def test_bf16_union_of_codes_maximum_heads_and_micro_batches():
    """64 heads (bit 63 of the per-micro-batch masks) and one image per micro-batch at 256 tokens."""
    w = di.Workload("mb_union_h64", 3, 40, 64, 64, 64, 64, 1, "bf16")
    rng = np.random.default_rng(87)
    ops_mb = [list(rng.choice([FULL, FWD, SKIP], size=64)) for _ in range(3)]
    ops_mb[0][63], ops_mb[1][63], ops_mb[2][63] = FULL, SKIP, FWD
    run_mb(w, ops_mb, [1, 1, 1], seed=87)
    w2 = di.Workload("mb_union_t256", 2, 256, 128, 2, 64, 256, 1, "bf16")
    run_mb(w2, [[FULL, SKIP], [FWD, FULL]], [1, 1], seed=88)


def test_bad_micro_batch_sizes_are_rejected():
    import paper_2504_12471_amd as P
    w = di.WORKLOADS["vit_tiny_fp32"]
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype)
    assert P.d2ft_block_saved_bytes_mb(desc, [1, 1]) == 0          # does not add up to the batch
    assert P.d2ft_block_saved_bytes_mb(desc, [4, 0]) == 0
    assert P.d2ft_block_saved_bytes_mb(desc, [2, 2]) > 0
