"""Caller-side loop over the blocks of a stack: buffer allocation and the two
sequences of d2ft_block_fwd / d2ft_block_bwd calls.  All arithmetic happens
inside the library; this file only owns device memory (torch tensors).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def torch_dtype(dtype: str) -> torch.dtype:
    return torch.float32 if dtype == "f32" else torch.bfloat16


def make_desc(batch: int, tokens: int, width: int, heads: int, mlp_hidden: int, dtype: str,
              lora_rank: int = 0, lora_scale: float = 1.0, ln_eps: float = 1e-6, head_dim: int = 64,
              flags: int = 0) -> B.BlockDesc:
    return B.BlockDesc(batch, tokens, width, heads, head_dim, mlp_hidden, lora_rank, ln_eps, lora_scale,
                       B.F32 if dtype == "f32" else B.BF16, flags)


def to_device(a: Optional[np.ndarray], dtype: str) -> Optional[torch.Tensor]:
    """Host fp32 array (already on the bf16 grid for bf16 workloads) -> contiguous device tensor."""
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda").to(torch_dtype(dtype)).contiguous()


class BlockStack:
    """L blocks with their weights on the device, one saved buffer per block, one scratch buffer."""

    def __init__(self, desc: B.BlockDesc, weights: List[Dict[str, Optional[torch.Tensor]]], dtype: str,
                 grad_fields: Optional[Sequence[str]] = None, mb_images: Optional[Sequence[int]] = None):
        """mb_images: images per micro-batch; when given, ops passed to forward/backward are
        [L][n_micro][heads] and every block call goes through the micro-batch entry points."""
        self.desc = desc
        # the backward calls of a pass follow each other: each leaves its weight-gradient work to be joined by the
        # next one, and backward() joins the last
        self.desc_bwd = B.BlockDesc.from_buffer_copy(desc)
        self.desc_bwd.flags |= B.FLAG_DEFER_JOIN
        self.mb_images = None if mb_images is None else [int(b) for b in mb_images]
        self.dtype = dtype
        self.weights = weights
        self.L = len(weights)
        tdt = torch_dtype(dtype)
        sb = (B.d2ft_block_saved_bytes(desc) if self.mb_images is None
              else B.d2ft_block_saved_bytes_mb(desc, self.mb_images))
        wb = B.d2ft_block_scratch_bytes(desc)
        if sb == 0 or wb == 0:
            raise B.D2ftError(B.ESHAPE, "descriptor rejected")
        self.saved = [torch.empty(sb, dtype=torch.uint8, device="cuda") for _ in range(self.L)]
        self.scratch = torch.empty(wb, dtype=torch.uint8, device="cuda")
        shape = (desc.batch, desc.tokens, desc.width)
        # hidden states between blocks: acts[l] is the input of block l, acts[L] the output
        self.acts = [None] + [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(self.L)]
        self.dacts = [torch.empty(shape, dtype=tdt, device="cuda") for _ in range(2)]
        if grad_fields is None:
            grad_fields = [k for k in B.WEIGHT_FIELDS if not k.startswith("ln")]
        self.grads = [{k: (torch.zeros_like(w[k]) if (k in grad_fields and w.get(k) is not None) else None)
                       for k in B.WEIGHT_FIELDS} for w in weights]

    def forward(self, x: torch.Tensor, ops: np.ndarray, stream=None) -> torch.Tensor:
        self.acts[0] = x
        for l in range(self.L):
            if self.mb_images is None:
                B.d2ft_block_fwd(self.desc, self.weights[l], ops[l], self.acts[l], self.acts[l + 1], self.saved[l],
                                 self.scratch, stream)
            else:
                B.d2ft_block_fwd_mb(self.desc, self.weights[l], self.mb_images, ops[l], self.acts[l], self.acts[l + 1],
                                    self.saved[l], self.scratch, stream)
        return self.acts[self.L]

    def backward(self, dy: torch.Tensor, ops: np.ndarray, stream=None) -> torch.Tensor:
        cur = dy
        for l in range(self.L - 1, -1, -1):
            out = self.dacts[l & 1]
            if self.mb_images is None:
                B.d2ft_block_bwd(self.desc_bwd, self.weights[l], ops[l], self.acts[l], cur, out, self.grads[l],
                                 self.saved[l], self.scratch, stream)
            else:
                B.d2ft_block_bwd_mb(self.desc_bwd, self.weights[l], self.mb_images, ops[l], self.acts[l], cur, out,
                                    self.grads[l], self.saved[l], self.scratch, stream)
            cur = out
        B.d2ft_join(stream)   # the gradients are complete on the stream when this returns
        return cur

    def step(self, x: torch.Tensor, dy: torch.Tensor, ops: np.ndarray, stream=None):
        """One pass of the whole hot path: forward through all blocks, then backward."""
        y = self.forward(x, ops, stream)
        dx = self.backward(dy, ops, stream)
        return y, dx
