"""Pins for the oracle's two subnets outside the blocks (Sec. IV-A: patch embedding; pooling + classifier).  No GPU.

  * the patch projection is a strided convolution: torch.nn.functional.conv2d (library routine) with the weight
    reshaped to [D, C, P, P], tokens in row-major patch order;
  * gradients of both subnets against torch autograd (conv2d / layer_norm / linear / cross_entropy);
  * a worked case: uniform logits give loss = log(n_classes); one-hot-confident logits give ~0.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import d2ft_oracle as orc
from test_oracle_block import relerr


def draw_embed(seed, B=3, C=3, H=12, W=8, P=4, D=10):
    rng = np.random.default_rng(seed)
    T = 1 + (H // P) * (W // P)
    return dict(images=rng.standard_normal((B, C, H, W)), w_pe=rng.standard_normal((D, C * P * P)),
                b_pe=rng.standard_normal(D), cls=rng.standard_normal(D), pos=rng.standard_normal((T, D)), P=P)


def torch_embed(e):
    t = {k: torch.tensor(v, requires_grad=(k != "images")) for k, v in e.items() if k != "P"}
    D, P = e["w_pe"].shape[0], e["P"]
    C = e["images"].shape[1]
    y = F.conv2d(t["images"], t["w_pe"].reshape(D, C, P, P), t["b_pe"], stride=P)        # [B, D, ny, nx]
    y = y.flatten(2).transpose(1, 2)                                                    # [B, ny*nx, D]
    tok = torch.cat([t["cls"].expand(y.shape[0], 1, D), y], dim=1) + t["pos"]
    return tok, t


def test_patch_embedding_is_a_strided_convolution():
    e = draw_embed(101)
    tok, _ = orc.patch_embed_fwd(e["images"], e["w_pe"], e["b_pe"], e["cls"], e["pos"], e["P"])
    ref, _ = torch_embed(e)
    assert relerr(tok, ref.detach().numpy()) < 1e-13


def test_patch_embedding_gradients_match_autograd():
    e = draw_embed(102)
    _, cache = orc.patch_embed_fwd(e["images"], e["w_pe"], e["b_pe"], e["cls"], e["pos"], e["P"])
    dtok = np.random.default_rng(103).standard_normal((3, 7, 10))
    g = orc.patch_embed_bwd(cache, dtok)
    ref, t = torch_embed(e)
    ref.backward(torch.tensor(dtok))
    for k in ("w_pe", "b_pe", "cls", "pos"):
        assert relerr(g[k], t[k].grad.numpy()) < 1e-12, k


def draw_head(seed, B=5, T=4, D=12, n=6):
    rng = np.random.default_rng(seed)
    return dict(tokens=rng.standard_normal((B, T, D)), ln_g=1 + 0.3 * rng.standard_normal(D), ln_b=rng.standard_normal(D),
                w_c=rng.standard_normal((n, D)), b_c=rng.standard_normal(n)), rng.integers(0, n, size=B)


def test_classifier_loss_and_gradients_match_autograd():
    h, labels = draw_head(104)
    loss, logits, cache = orc.classifier_fwd(h["tokens"], h["ln_g"], h["ln_b"], h["w_c"], h["b_c"], labels)
    dtok, g = orc.classifier_bwd(cache)
    t = {k: torch.tensor(v, requires_grad=True) for k, v in h.items()}
    z = F.linear(F.layer_norm(t["tokens"][:, 0], (12,), t["ln_g"], t["ln_b"], 1e-6), t["w_c"], t["b_c"])
    ref = F.cross_entropy(z, torch.tensor(labels))
    ref.backward()
    assert abs(loss - float(ref)) < 1e-13 and relerr(logits, z.detach().numpy()) < 1e-13
    assert relerr(dtok, t["tokens"].grad.numpy()) < 1e-12
    assert np.all(dtok[:, 1:] == 0.0)
    for k in ("ln_g", "ln_b", "w_c", "b_c"):
        assert relerr(g[k], t[k].grad.numpy()) < 1e-12, k


def test_uniform_and_confident_logits():
    h, labels = draw_head(105)
    h["w_c"][:] = 0.0
    h["b_c"][:] = 0.7
    loss, _, _ = orc.classifier_fwd(h["tokens"], h["ln_g"], h["ln_b"], h["w_c"], h["b_c"], labels)
    assert abs(loss - np.log(6)) < 1e-14
    h["b_c"][:] = 0.0
    big = np.zeros((5, 6)); big[np.arange(5), labels] = 50.0
    # logits that do not depend on the input: put them in through the bias of a one-image batch each
    for b in range(5):
        hb = {k: v for k, v in h.items()}
        hb["b_c"] = big[b]
        l, _, _ = orc.classifier_fwd(h["tokens"][b:b + 1], h["ln_g"], h["ln_b"], h["w_c"], hb["b_c"], labels[b:b + 1])
        assert 0.0 <= l < 1e-20
