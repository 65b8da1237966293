"""GPU parity: libd2ft (through its C ABI) against the CPU fp64 oracle, element by element.

Bar: bit-exact for op-code work (compaction, knapsack, zero gradient slices); per tensor
max|gpu - oracle| / max|oracle| <= 1e-4 (fp32) or 2e-2 (bf16 storage, fp32 accumulate).
For bf16 workloads the oracle consumes the bf16-rounded inputs promoted to fp64.
"""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import TOL, compare_block, gpu_block, oracle_block, rel_inf

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


def draw_block(w, seed):
    rng = np.random.default_rng(seed)
    x = di.draw_hidden(rng, w)
    wt = di.draw_block_weights(rng, w)
    dy = di.draw_hidden(rng, w)
    return x, wt, dy


def run_case(w, ops, seed=0, flags=0, grad_fields=None, tol=None):
    x, wt, dy = draw_block(w, seed)
    fields = di.WEIGHT_FIELDS if grad_fields is None else grad_fields
    got = gpu_block(w, wt, ops, x, dy, fields, flags)
    ref = oracle_block(w, wt, ops, x, dy)
    rep = {}
    compare_block(w, ops, got, ref, TOL[w.dtype] if tol is None else tol, fields, rep)
    print(f"[{w.name} ops={list(ops)} flags={flags}] " + " ".join(f"{k}={v:.2e}" for k, v in rep.items()), flush=True)
    return got, ref


# ---------------------------------------------------------------------------
# configuration 1: ViT-Tiny-shaped fp32 block, mask [full, fwd-only, skip]
# ---------------------------------------------------------------------------
def test_vit_tiny_fp32_block():
    w = di.WORKLOADS["vit_tiny_fp32"]
    run_case(w, [FULL, FWD, SKIP])


@pytest.mark.parametrize("ops", [(FULL, FULL, FULL), (SKIP, SKIP, SKIP), (FWD, FWD, FWD), (SKIP, FWD, FULL),
                                 (FWD, SKIP, SKIP), (SKIP, FULL, SKIP)])
def test_fp32_masks(ops):
    w = di.WORKLOADS["vit_tiny_fp32"]
    run_case(w, list(ops), seed=1)


def test_fp32_all_skip_is_residual_plus_mlp_bitwise():
    """All-shortcut block: x1 is x itself, so y equals the all-skip run of a block with different attention weights."""
    w = di.WORKLOADS["vit_tiny_fp32"]
    x, wt, dy = draw_block(w, 2)
    y1, dx1, _ = gpu_block(w, wt, [SKIP] * 3, x, dy)
    wt2 = dict(wt)
    rng = np.random.default_rng(99)
    for k in ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b"):
        wt2[k] = (rng.standard_normal(wt[k].shape) * 0.5).astype(np.float32)
    y2, dx2, _ = gpu_block(w, wt2, [SKIP] * 3, x, dy)
    assert np.array_equal(y1, y2) and np.array_equal(dx1, dx2)


# ragged shapes: token count and widths that are not multiples of the tile sizes
RAGGED = di.Workload("ragged_f32", 3, 37, 72, 5, 64, 136, 1, "f32")


@pytest.mark.parametrize("ops", [(FULL, SKIP, FWD, FULL, FWD), (FWD, FULL, SKIP, SKIP, SKIP), (FULL,) * 5])
def test_fp32_ragged(ops):
    run_case(RAGGED, list(ops), seed=3)


def test_single_token_single_head():
    w = di.Workload("one", 1, 1, 64, 1, 64, 8, 1, "f32")
    run_case(w, [FULL], seed=4)


def test_null_bias_and_frozen_fields():
    w = di.WORKLOADS["vit_tiny_fp32"]
    x, wt, dy = draw_block(w, 5)
    wt["b_o"] = None
    wt["b2"] = None
    fields = ("w_qkv", "w_o", "w1", "b1")
    ops = [FULL, FWD, FULL]
    got = gpu_block(w, wt, ops, x, dy, fields)
    ref = oracle_block(w, wt, ops, x, dy)
    compare_block(w, ops, got, ref, TOL["f32"], fields)
    assert got[2]["b_qkv"] is None and got[2]["w2"] is None


def test_accumulate_mode_adds_and_leaves_non_full_slices():
    w = di.WORKLOADS["vit_tiny_fp32"]
    x, wt, dy = draw_block(w, 6)
    ops = [FULL, FWD, SKIP]
    rng = np.random.default_rng(7)
    init = {k: (rng.standard_normal(v.shape) * 0.1).astype(np.float32) for k, v in wt.items() if v is not None}
    _, _, g = gpu_block(w, wt, ops, x, dy, di.WEIGHT_FIELDS, flags=1, grads_init=init)
    _, _, rg, _ = oracle_block(w, wt, ops, x, dy)
    for k, v in g.items():
        if v is None:
            continue
        assert rel_inf(v, init[k] + rg[k]) < 1e-4, k
    dh = w.head_dim
    for h in (1, 2):   # not p_f: untouched, bit for bit
        assert np.array_equal(g["w_qkv"][:, h], init["w_qkv"][:, h])
        assert np.array_equal(g["b_qkv"][:, h], init["b_qkv"][:, h])
        assert np.array_equal(g["w_o"][:, h * dh:(h + 1) * dh], init["w_o"][:, h * dh:(h + 1) * dh])


# ---------------------------------------------------------------------------
# LoRA (Sec. II-D)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_lora_block(dtype):
    w = di.Workload("lora_" + dtype, 2, 33, 128, 4, 64, 256, 1, dtype, lora_rank=8, lora_scale=1.5,
                    lora_b_zero=False)
    run_case(w, [FULL, SKIP, FWD, FULL], seed=8)


def test_lora_zero_b_and_frozen_base():
    w = di.Workload("lora_frozen", 2, 33, 128, 4, 64, 256, 1, "f32", lora_rank=8, lora_b_zero=True)
    fields = ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v")
    got, ref = run_case(w, [FULL, FULL, SKIP, FWD], seed=9, grad_fields=fields)
    assert np.all(got[2]["lora_a_q"] == 0.0) and np.all(got[2]["lora_a_v"] == 0.0)


# ---------------------------------------------------------------------------
# bf16: both kernel families
# ---------------------------------------------------------------------------
SMALL_BF16 = di.Workload("small_bf16", 3, 70, 256, 4, 64, 512, 1, "bf16")
MID_BF16 = di.Workload("mid_bf16", 5, 197, 384, 6, 64, 1536, 1, "bf16")   # ViT-Small block: several tiles + ragged tails


@pytest.mark.parametrize("flags", [0, 2])
@pytest.mark.parametrize("ops", [(FULL, FWD, SKIP, FULL), (FULL,) * 4, (SKIP,) * 4, (FWD, FWD, SKIP, FWD)])
def test_bf16_small(ops, flags):
    run_case(SMALL_BF16, list(ops), seed=10, flags=flags)


@pytest.mark.parametrize("flags", [0, 2])
def test_bf16_vit_small_block(flags):
    run_case(MID_BF16, [FULL, FWD, SKIP, FULL, FULL, FWD], seed=11, flags=flags)


def test_bf16_key_bias_gradient_is_exactly_zero():
    """The matrix-core attention backward writes the key-bias gradient as the zero it is (softmax does not see
    a common shift of the keys; pinned for the oracle in test_oracle_block.py) instead of adding up rounded
    dK rows; the value and query planes of the same tensor are compared with the oracle by run_case."""
    ops = [FULL, FWD, SKIP, FULL, FULL, FWD]
    got, _ = run_case(MID_BF16, ops, seed=13)
    gb = np.asarray(got[2]["b_qkv"], dtype=np.float64).reshape(3, MID_BF16.heads, 64)
    for h, o in enumerate(ops):
        if o == FULL:
            assert np.all(gb[1, h] == 0.0)
            assert np.abs(gb[0, h]).max() > 0.0 and np.abs(gb[2, h]).max() > 0.0


def test_bf16_ragged_widths():
    w = di.Workload("ragged_bf16", 2, 50, 200, 3, 64, 328, 1, "bf16")
    run_case(w, [FWD, FULL, FULL], seed=12)


# ---------------------------------------------------------------------------
# stack of blocks
# ---------------------------------------------------------------------------
def test_small_stack_against_oracle():
    import torch
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    w = di.Workload("stack_bf16", 4, 50, 256, 4, 64, 512, 3, "bf16", mask=("counts", 0.5, 0.25, 0.25))
    s = di.draw_stack(w, seed=13)
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype)
    dws = [{k: P.to_device(v, w.dtype) for k, v in bw.items()} for bw in s.weights]
    st = P.BlockStack(desc, dws, w.dtype)
    y, dx = st.step(P.to_device(s.x, w.dtype), P.to_device(s.dy, w.dtype), s.ops)
    torch.cuda.synchronize()
    ry, caches = orc.stack_fwd(s.weights, s.ops, s.x, w.head_dim)
    rdx, rgrads = orc.stack_bwd(s.weights, caches, s.dy)
    assert rel_inf(y.float().cpu().numpy(), ry) < 2e-2
    assert rel_inf(dx.float().cpu().numpy(), rdx) < 2e-2
    for l in range(w.blocks):
        for k in ("w_qkv", "w_o", "w1", "w2", "b1"):
            assert rel_inf(st.grads[l][k].float().cpu().numpy(), rgrads[l][k]) < 2e-2, (l, k)


# ---------------------------------------------------------------------------
# limits of the supported shapes
# ---------------------------------------------------------------------------
def test_bf16_tokens_beyond_the_matrix_core_attention_limit():
    """More than 256 tokens: the bf16 block takes the vector-ALU attention kernels, GEMMs stay on the matrix cores."""
    w = di.Workload("long_bf16", 1, 300, 128, 2, 64, 256, 1, "bf16")
    run_case(w, [FULL, FWD], seed=14)


def test_bf16_exactly_256_tokens_and_one_token_tail():
    run_case(di.Workload("t256_bf16", 2, 256, 128, 2, 64, 256, 1, "bf16"), [FULL, FULL], seed=15)
    run_case(di.Workload("t225_bf16", 2, 225, 128, 2, 64, 256, 1, "bf16"), [FULL, SKIP], seed=16)   # 7 tiles + 1 token


def test_maximum_head_count():
    w = di.Workload("h64_f32", 1, 9, 64, 64, 64, 64, 1, "f32")
    rng = np.random.default_rng(17)
    ops = list(rng.choice([FULL, FWD, SKIP], size=64))
    run_case(w, ops, seed=17)
    wb = di.Workload("h64_bf16", 1, 40, 64, 64, 64, 64, 1, "bf16")
    run_case(wb, ops, seed=18)


def test_unsupported_shapes_are_rejected_without_a_launch():
    import paper_2504_12471_amd as P
    for kw in (dict(batch=0), dict(tokens=0), dict(tokens=1025), dict(width=12), dict(heads=65), dict(head_dim=32),
               dict(mlp_hidden=4)):
        base = dict(batch=1, tokens=8, width=64, heads=2, mlp_hidden=64, dtype="f32", head_dim=64)
        base.update(kw)
        desc = P.make_desc(base["batch"], base["tokens"], base["width"], base["heads"], base["mlp_hidden"], base["dtype"],
                           0, 1.0, 1e-6, base["head_dim"])
        assert P.d2ft_block_saved_bytes(desc) == 0 and P.d2ft_block_scratch_bytes(desc) == 0, kw


def test_one_stream_and_second_stream_agree():
    """The backward's weight-gradient launches run on a second stream of the library by default and on the
    caller's with D2FT_FLAG_ONE_STREAM: same y and dx bit for bit, gradients to rounding order (the two modes group
    the weight gradients into launches differently), both against the oracle; the two-stream call is repeated to
    show that a call does not disturb the next one."""
    FLAG_ONE_STREAM = 8
    ops = [FULL, FWD, SKIP, FULL, FULL, FWD]
    x, wt, dy = draw_block(MID_BF16, 21)
    one = gpu_block(MID_BF16, wt, ops, x, dy, di.WEIGHT_FIELDS, FLAG_ONE_STREAM)
    two = gpu_block(MID_BF16, wt, ops, x, dy, di.WEIGHT_FIELDS, 0)
    again = gpu_block(MID_BF16, wt, ops, x, dy, di.WEIGHT_FIELDS, 0)
    ref = oracle_block(MID_BF16, wt, ops, x, dy)
    for got in (one, two):
        compare_block(MID_BF16, ops, got, ref, TOL["bf16"], di.WEIGHT_FIELDS)
    assert np.array_equal(one[0], two[0]) and np.array_equal(one[1], two[1])
    for k, v in two[2].items():
        if v is not None:
            assert np.array_equal(v, again[2][k]), k
            assert rel_inf(v, np.asarray(one[2][k], np.float64)) <= 2.0 ** -7, k


def test_block_calls_captured_in_a_hip_graph():
    """Forward + backward captured from a stream: the library then keeps every launch on that stream (no second
    stream, no event of its own in the graph).  Every replay, with eager work and synchronisations in between,
    must give what the eager calls gave."""
    import torch
    import paper_2504_12471_amd as P
    w, ops = MID_BF16, [FULL, FWD, SKIP, FULL, FULL, FWD]
    x, wt, dy = draw_block(w, 22)
    desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype)
    dw = {k: P.to_device(v, w.dtype) for k, v in wt.items()}
    xd, dyd = P.to_device(x, w.dtype), P.to_device(dy, w.dtype)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    saved = torch.empty(P.d2ft_block_saved_bytes(desc), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(P.d2ft_block_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    grads = {k: (None if v is None else torch.zeros_like(v)) for k, v in dw.items()}

    def calls():
        P.d2ft_block_fwd(desc, dw, ops, xd, y, saved, scratch)
        P.d2ft_block_bwd(desc, dw, ops, xd, dyd, dx, grads, saved, scratch)

    def poison():
        y.fill_(float("nan"))
        dx.fill_(float("nan"))
        for v in grads.values():
            if v is not None:
                v.fill_(float("nan"))

    calls()
    torch.cuda.synchronize()
    eager = (y.clone(), dx.clone(), {k: (None if v is None else v.clone()) for k, v in grads.items()})
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for _ in range(3):
        poison()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, eager[0]) and torch.equal(dx, eager[1])
        for k, v in grads.items():
            if v is not None:
                assert rel_inf(v.float().cpu().numpy(), eager[2][k].double().cpu().numpy()) <= 2.0 ** -7, k
        calls()   # eager work between the replays
        torch.cuda.synchronize()


def test_deferred_join_over_consecutive_backward_calls():
    """Backward calls of two blocks in a row with D2FT_FLAG_DEFER_JOIN: the second call takes over the wait for the
    first one's weight gradients, d2ft_join (or the next call into the library) orders the rest on the stream.
    Against the same calls without the flag, bit for bit (the launches are the same); only the caller's stream is
    synchronised before the results are read."""
    import torch
    import paper_2504_12471_amd as P
    w = MID_BF16   # 24 feed-forward gradient tiles: they go to the second stream on their own
    ops = [[FULL, FWD, SKIP, FULL, FULL, FWD], [FULL, FULL, FWD, SKIP, FULL, FULL]]
    rng = np.random.default_rng(23)
    x, dy = di.draw_hidden(rng, w), di.draw_hidden(rng, w)
    wts = [di.draw_block_weights(rng, w) for _ in range(2)]
    dws = [{k: P.to_device(v, w.dtype) for k, v in wt.items()} for wt in wts]
    xd, dyd = P.to_device(x, w.dtype), P.to_device(dy, w.dtype)

    def run(flags, finish):
        desc = P.make_desc(w.batch, w.tokens, w.width, w.heads, w.mlp_hidden, w.dtype, 0, 1.0, w.ln_eps, w.head_dim, flags)
        saved = [torch.empty(P.d2ft_block_saved_bytes(desc), dtype=torch.uint8, device="cuda") for _ in range(2)]
        scratch = torch.empty(P.d2ft_block_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
        h = [xd, torch.empty_like(xd), torch.empty_like(xd)]
        d = [torch.empty_like(xd), torch.empty_like(xd), dyd]
        grads = [{k: (None if v is None else torch.full_like(v, float("nan"))) for k, v in dw.items()} for dw in dws]
        for l in range(2):
            P.d2ft_block_fwd(desc, dws[l], ops[l], h[l], h[l + 1], saved[l], scratch)
        for l in (1, 0):
            P.d2ft_block_bwd(desc, dws[l], ops[l], h[l], d[l + 1], d[l], grads[l], saved[l], scratch)
        finish(desc, h, saved, scratch)
        torch.cuda.current_stream().synchronize()
        return d[0].clone(), [{k: (None if v is None else v.clone()) for k, v in g.items()} for g in grads]

    plain = run(0, lambda *a: None)
    joined = run(P.FLAG_DEFER_JOIN, lambda *a: P.d2ft_join())
    # no explicit join: the next call into the library (a forward call into spare buffers) waits first
    spare_y = torch.empty_like(xd)
    by_next_call = run(P.FLAG_DEFER_JOIN,
                       lambda desc, h, saved, scratch: P.d2ft_block_fwd(desc, dws[0], ops[0], h[0], spare_y,
                                                                        torch.empty_like(saved[0]), scratch))
    for got in (joined, by_next_call):
        assert torch.equal(got[0], plain[0])
        for l in range(2):
            for k, v in plain[1][l].items():
                if v is not None:
                    assert torch.equal(got[1][l][k], v), (l, k)
