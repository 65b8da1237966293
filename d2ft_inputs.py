"""Seeded synthetic inputs for the head-selective ViT block path.

This module only *draws* data: hidden states, block weights, upstream
gradients, per-head operation masks and knapsack utilities.  It holds none of
the method's arithmetic, and it is the only module that both the CPU oracle's
tests and the HIP path's tests / benchmark import.

Shapes follow the paper's workload (Sec. III-A "Model": 224x224 images, patch
16 -> 196 patches + CLS = 197 tokens; pre-LN ViT blocks with H heads and a
two-layer feed-forward network).  The paper's datasets are replaced by
N(0,1) token batches: throughput and numerics of the block do not depend on
pixel content.

Draw order for one workload: one numpy ``default_rng(seed)`` stream gives x,
then for each block its weights in the order of ``WEIGHT_FIELDS``, then dy.
The op-code mask (its permutation, or the two utility arrays of the knapsack)
comes from a stream of its own, ``default_rng([seed, MASK_STREAM])``, so that
it does not depend on the batch size or on any other shape: a test that draws a
smaller batch gets the same op codes as the benchmark.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

# Operation codes of the scheduling table (Alg. 1: 1 = p_f, 2 = p_o, 3 = p_s).
OP_FULL, OP_FWD, OP_SKIP = 1, 2, 3

WEIGHT_FIELDS = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
    "w1", "b1", "w2", "b2", "lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v",
)


@dataclass(frozen=True)
class Workload:
    """One configuration: block shape, depth, storage dtype and mask recipe."""
    name: str
    batch: int
    tokens: int
    width: int
    heads: int            # heads held by this device (may be a share of the model's)
    head_dim: int
    mlp_hidden: int
    blocks: int
    dtype: str            # "f32" or "bf16" (storage; accumulation is fp32 on the GPU)
    lora_rank: int = 0
    lora_scale: float = 1.0
    ln_eps: float = 1e-6
    # mask recipe: ("fixed", [codes]) | ("counts", frac_full, frac_fwd, frac_skip) | ("knapsack", capacity_fraction)
    mask: tuple = ("counts", 1.0, 0.0, 0.0)
    lora_b_zero: bool = True
    train_base: bool = True   # False: base weights frozen, only LoRA gradients wanted
    gate_ffn: bool = False    # True: a head's op code also governs its 1/H slice of the feed-forward network

    @property
    def rows(self) -> int:
        return self.batch * self.tokens


WORKLOADS: Dict[str, Workload] = {
    # single ViT-Tiny-shaped block, fp32, mask [full, fwd-only, skip]
    "vit_tiny_fp32": Workload("vit_tiny_fp32", 4, 65, 192, 3, 64, 768, 1, "f32",
                              mask=("fixed", [OP_FULL, OP_FWD, OP_SKIP])),
    # ViT-B/16 stack, 60% full / 20% fwd-only / 20% skip
    "vit_b16": Workload("vit_b16", 64, 197, 768, 12, 64, 3072, 12, "bf16",
                        mask=("counts", 0.6, 0.2, 0.2)),
    # ViT-B/16 with 40% of the heads skipped and no forward-only heads
    "vit_b16_skip40": Workload("vit_b16_skip40", 64, 197, 768, 12, 64, 3072, 12, "bf16",
                               mask=("counts", 0.6, 0.0, 0.4)),
    # one device's share of ViT-B/16: 4 of 12 heads and 1/3 of the MLP per block
    "vit_b16_share4": Workload("vit_b16_share4", 64, 197, 768, 4, 64, 1024, 12, "bf16",
                               mask=("knapsack", 0.6)),
    # ViT-L/16 stack, 40% skipped, 20% fwd-only
    "vit_l16": Workload("vit_l16", 32, 197, 1024, 16, 64, 4096, 24, "bf16",
                        mask=("counts", 0.4, 0.2, 0.4)),
    # the ViT-B/16 stack with whole subnets gated (head + 1/12 of the FFN), same 60/20/20 mask
    "vit_b16_ffn": Workload("vit_b16_ffn", 64, 197, 768, 12, 64, 3072, 12, "bf16",
                            mask=("counts", 0.6, 0.2, 0.2), gate_ffn=True),
    # the same with 40% of the subnets skipped and no forward-only ones
    "vit_b16_ffn_skip40": Workload("vit_b16_ffn_skip40", 64, 197, 768, 12, 64, 3072, 12, "bf16",
                                   mask=("counts", 0.6, 0.0, 0.4), gate_ffn=True),
    # ViT-B/16 with rank-8 LoRA on Wq and Wv, base frozen, 40% skipped
    "vit_b16_lora": Workload("vit_b16_lora", 64, 197, 768, 12, 64, 3072, 12, "bf16",
                             lora_rank=8, mask=("counts", 0.6, 0.0, 0.4), train_base=False),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller batch, fewer blocks ...)."""
    return replace(w, **kw)


# ----------------------------------------------------------------------------
# bf16 grid helpers (data preparation only)
# ----------------------------------------------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round an fp32 array to the nearest bf16 value (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """The upper 16 bits of an fp32 array that already lies on the bf16 grid."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
def draw_hidden(rng: np.random.Generator, w: Workload) -> np.ndarray:
    """Hidden states or upstream gradient: N(0,1), shape [batch, tokens, width]."""
    return _store(rng.standard_normal((w.batch, w.tokens, w.width)), w.dtype)


def draw_block_weights(rng: np.random.Generator, w: Workload) -> Dict[str, Optional[np.ndarray]]:
    """Weights of one block in WEIGHT_FIELDS order.

    Matrices and biases are N(0, 0.02^2); LayerNorm scale is 1 + N(0, 0.02^2).
    LoRA A is N(0, 0.02^2); LoRA B is zero when ``lora_b_zero`` else N(0, 0.02^2).
    Layouts: w_qkv [3, heads, head_dim, width]; b_qkv [3, heads, head_dim];
    w_o [width, heads*head_dim]; w1 [mlp, width]; w2 [width, mlp];
    lora_a_* [heads, r, width]; lora_b_* [heads, head_dim, r].
    """
    D, H, dh, Dm, r = w.width, w.heads, w.head_dim, w.mlp_hidden, w.lora_rank
    s = 0.02
    n = lambda *shape: rng.standard_normal(shape) * s
    out: Dict[str, Optional[np.ndarray]] = {}
    out["ln1_g"] = 1.0 + n(D)
    out["ln1_b"] = n(D)
    out["w_qkv"] = n(3, H, dh, D)
    out["b_qkv"] = n(3, H, dh)
    out["w_o"] = n(D, H * dh)
    out["b_o"] = n(D)
    out["ln2_g"] = 1.0 + n(D)
    out["ln2_b"] = n(D)
    out["w1"] = n(Dm, D)
    out["b1"] = n(Dm)
    out["w2"] = n(D, Dm)
    out["b2"] = n(D)
    if r > 0:
        out["lora_a_q"] = n(H, r, D)
        out["lora_a_v"] = n(H, r, D)
        bq, bv = n(H, dh, r), n(H, dh, r)
        if w.lora_b_zero:
            bq, bv = np.zeros_like(bq), np.zeros_like(bv)
        out["lora_b_q"], out["lora_b_v"] = bq, bv
    else:
        for k in ("lora_a_q", "lora_a_v", "lora_b_q", "lora_b_v"):
            out[k] = None
    return {k: (None if v is None else _store(v, w.dtype)) for k, v in out.items()}


def exact_count_masks(rng: np.random.Generator, blocks: int, heads: int,
                      frac_full: float, frac_fwd: float, frac_skip: float) -> np.ndarray:
    """uint8 [blocks, heads] op codes with exact global counts, placed by a seeded shuffle.

    Counts over all blocks*heads heads: fwd-only and skip are rounded to nearest,
    the remainder is full.
    """
    total = blocks * heads
    n_fwd = int(np.floor(frac_fwd * total + 0.5))
    n_skip = int(np.floor(frac_skip * total + 0.5))
    n_full = total - n_fwd - n_skip
    assert n_full >= 0 and abs(frac_full + frac_fwd + frac_skip - 1.0) < 1e-9
    codes = np.array([OP_FULL] * n_full + [OP_FWD] * n_fwd + [OP_SKIP] * n_skip, dtype=np.uint8)
    return codes[rng.permutation(total)].reshape(blocks, heads)


@dataclass
class KnapsackInputs:
    """Inputs of the bi-level knapsack selection (Alg. 1 inputs), all host arrays."""
    score_full: np.ndarray   # [K, n] float64, backward contribution scores
    score_fwd: np.ndarray    # [K, n] float64, forward contribution scores
    cost_fwd: np.ndarray     # [K] int32
    cost_bwd: np.ndarray     # [K] int32
    cap_full: np.ndarray     # [K] int32
    cap_fwd: np.ndarray      # [K] int32


def draw_knapsack_inputs(rng: np.random.Generator, n_knapsacks: int, n_items: int,
                         cost_fwd: int = 1, cost_bwd: int = 2,
                         capacity_fraction: float = 0.6) -> KnapsackInputs:
    """Two independent U(0,1) utility arrays and a budget split.

    The total budget is floor(capacity_fraction * all-full cost).  The full
    stage gets all of it; the forward-only stage gets what cannot buy another
    full item.
    """
    sf = rng.random((n_knapsacks, n_items))
    so = rng.random((n_knapsacks, n_items))
    full_cost = cost_fwd + cost_bwd
    budget = int(np.floor(capacity_fraction * full_cost * n_items + 1e-9))
    n_full = budget // full_cost
    cap_full = budget
    cap_fwd = budget - n_full * full_cost
    K = n_knapsacks
    return KnapsackInputs(
        score_full=sf, score_fwd=so,
        cost_fwd=np.full(K, cost_fwd, np.int32), cost_bwd=np.full(K, cost_bwd, np.int32),
        cap_full=np.full(K, cap_full, np.int32), cap_fwd=np.full(K, cap_fwd, np.int32))


@dataclass
class StackInputs:
    workload: Workload
    x: np.ndarray                       # [B, T, D] fp32 values (on the bf16 grid when dtype is bf16)
    weights: List[Dict[str, Optional[np.ndarray]]]
    dy: np.ndarray
    ops: Optional[np.ndarray]           # uint8 [blocks, heads]; None when the mask comes from the knapsack
    knapsack: Optional[KnapsackInputs] = None


MASK_STREAM = 0x6D61736B   # second word of the seed sequence of the op-code stream


def draw_ops(w: Workload, seed: int = 0) -> Tuple[Optional[np.ndarray], Optional[KnapsackInputs]]:
    """The workload's op codes [blocks, heads] (or, for a knapsack recipe, the selection's inputs), from
    their own seeded stream: they depend on blocks, heads and the recipe only."""
    rng = np.random.default_rng([seed, MASK_STREAM])
    kind = w.mask[0]
    if kind == "fixed":
        ops = np.tile(np.asarray(w.mask[1], dtype=np.uint8), (w.blocks, 1))
        assert ops.shape[1] == w.heads
        return ops, None
    if kind == "counts":
        return exact_count_masks(rng, w.blocks, w.heads, *w.mask[1:]), None
    if kind == "knapsack":
        return None, draw_knapsack_inputs(rng, 1, w.blocks * w.heads, 1, 2, w.mask[1])
    raise ValueError(kind)


def draw_stack(w: Workload, seed: int = 0) -> StackInputs:
    """All tensors of one workload, in the documented draw order."""
    rng = np.random.default_rng(seed)
    x = draw_hidden(rng, w)
    weights = [draw_block_weights(rng, w) for _ in range(w.blocks)]
    dy = draw_hidden(rng, w)
    ops, ks = draw_ops(w, seed)
    return StackInputs(w, x, weights, dy, ops, ks)


def all_full_ops(w: Workload) -> np.ndarray:
    return np.full((w.blocks, w.heads), OP_FULL, dtype=np.uint8)
