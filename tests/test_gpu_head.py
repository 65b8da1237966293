"""GPU parity for the two subnets outside the blocks (Sec. IV-A): d2ft_patch_embed_fwd / _bwd and
d2ft_classifier_fwd_bwd against the oracle.  Tolerances as for the blocks (1e-4 fp32, 2e-2 bf16 per
tensor, infinity-norm relative); the loss is fp32 arithmetic on exact inputs: 1e-5."""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import TOL, rel_inf

pytestmark = pytest.mark.gpu


def grid(a, dtype):
    a = np.asarray(a, np.float32)
    return di.round_to_bf16(a) if dtype == "bf16" else a


def run_embed(dtype, B, C, H, W, P, D, seed, accumulate=False):
    import torch
    import paper_2504_12471_amd as Pk
    from oracle import d2ft_oracle as orc
    rng = np.random.default_rng(seed)
    T = 1 + (H // P) * (W // P)
    K = C * P * P
    h = dict(images=grid(rng.standard_normal((B, C, H, W)), dtype), w_pe=grid(rng.standard_normal((D, K)) * 0.05, dtype),
             b_pe=grid(rng.standard_normal(D) * 0.1, dtype), cls=grid(rng.standard_normal(D), dtype),
             pos=grid(rng.standard_normal((T, D)) * 0.5, dtype))
    dtok = grid(rng.standard_normal((B, T, D)), dtype)
    desc = Pk.EmbedDesc(B, C, H, W, P, D, Pk.BF16 if dtype == "bf16" else Pk.F32, 1 if accumulate else 0)
    dev = {k: Pk.to_device(v, dtype) for k, v in h.items()}
    tokens = torch.empty((B, T, D), dtype=Pk.torch_dtype(dtype), device="cuda")
    saved = torch.empty(Pk.d2ft_embed_saved_bytes(desc), dtype=torch.uint8, device="cuda")
    scratch = torch.empty(Pk.d2ft_embed_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    Pk.d2ft_patch_embed_fwd(desc, dev["images"], dev["w_pe"], dev["b_pe"], dev["cls"], dev["pos"], tokens, saved, scratch)
    init = {k: grid(rng.standard_normal(h[k].shape) * 0.1, dtype) for k in ("w_pe", "b_pe", "cls", "pos")}
    g = {k: (Pk.to_device(init[k], dtype) if accumulate else torch.full_like(dev[k], float("nan"))) for k in init}
    Pk.d2ft_patch_embed_bwd(desc, Pk.to_device(dtok, dtype), g["w_pe"], g["b_pe"], g["cls"], g["pos"], saved, scratch)
    torch.cuda.synchronize()
    rtok, cache = orc.patch_embed_fwd(h["images"], h["w_pe"], h["b_pe"], h["cls"], h["pos"], P)
    rg = orc.patch_embed_bwd(cache, dtok)
    tol = TOL[dtype]
    errs = {"tokens": rel_inf(tokens.float().cpu().numpy(), rtok)}
    for k in init:
        ref = rg[k] + (init[k] if accumulate else 0.0)
        errs["d" + k] = rel_inf(g[k].float().cpu().numpy(), ref)
    print(f"[embed {dtype} B={B} {C}x{H}x{W} P={P} D={D}] " + " ".join(f"{k}={v:.1e}" for k, v in errs.items()), flush=True)
    assert all(v <= tol for v in errs.values()), errs


def test_embed_fp32_small():
    run_embed("f32", 3, 3, 32, 24, 8, 40, 111)


def test_embed_fp32_accumulate():
    run_embed("f32", 2, 1, 16, 16, 8, 16, 112, accumulate=True)


def test_embed_bf16_vit_shape():
    """The ViT-B/16 embedding at a small batch: 224 x 224 x 3 images, 16 x 16 patches, 197 tokens, D = 768."""
    run_embed("bf16", 4, 3, 224, 224, 16, 768, 113)


def run_head(dtype, B, T, D, n, seed, frozen_ln=False):
    import torch
    import paper_2504_12471_amd as Pk
    from oracle import d2ft_oracle as orc
    rng = np.random.default_rng(seed)
    h = dict(tokens=grid(rng.standard_normal((B, T, D)), dtype), ln_g=grid(1 + 0.2 * rng.standard_normal(D), dtype),
             ln_b=grid(0.1 * rng.standard_normal(D), dtype), w_c=grid(rng.standard_normal((n, D)) * 0.2, dtype),
             b_c=grid(rng.standard_normal(n) * 0.1, dtype))
    labels = rng.integers(0, n, size=B)
    desc = Pk.HeadDesc(B, T, D, n, 1e-6, Pk.BF16 if dtype == "bf16" else Pk.F32, 0)
    dev = {k: Pk.to_device(v, dtype) for k, v in h.items()}
    dtok = torch.full_like(dev["tokens"], float("nan"))
    g = {k: torch.full_like(dev[k], float("nan")) for k in ("ln_g", "ln_b", "w_c", "b_c")}
    if frozen_ln:
        g["ln_g"] = g["ln_b"] = None
    scratch = torch.empty(Pk.d2ft_head_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    loss = Pk.d2ft_classifier_fwd_bwd(desc, dev["tokens"], dev["ln_g"], dev["ln_b"], dev["w_c"], dev["b_c"], labels, dtok,
                                      g["ln_g"], g["ln_b"], g["w_c"], g["b_c"], scratch)
    rloss, _, cache = orc.classifier_fwd(h["tokens"], h["ln_g"], h["ln_b"], h["w_c"], h["b_c"], labels)
    rdtok, rg = orc.classifier_bwd(cache)
    tol = TOL[dtype]
    assert abs(loss - rloss) <= 1e-5 * max(1.0, abs(rloss)), (loss, rloss)
    got = dtok.float().cpu().numpy()
    assert np.all(got[:, 1:] == 0.0) and not np.any(np.signbit(got[:, 1:]))
    errs = {"dtokens": rel_inf(got, rdtok)}
    for k, t in g.items():
        if t is not None:
            errs["d" + k] = rel_inf(t.float().cpu().numpy(), rg[k])
    print(f"[head {dtype} B={B} T={T} D={D} n={n}] loss={loss:.6f} ref={rloss:.6f} " +
          " ".join(f"{k}={v:.1e}" for k, v in errs.items()), flush=True)
    assert all(v <= tol for v in errs.values()), errs


def test_head_fp32_small():
    run_head("f32", 5, 4, 24, 7, 121)


def test_head_bf16_vit_shape_100_classes():
    run_head("bf16", 64, 197, 768, 100, 122)


def test_head_frozen_norm_and_single_class_count_edge():
    run_head("f32", 2, 1, 8, 1, 123, frozen_ln=True)        # one class: loss 0, zero gradients
    run_head("f32", 3, 2, 16, 300, 124, frozen_ln=True)     # more classes than threads in a workgroup


def test_bad_labels_and_shapes_are_rejected():
    import torch
    import paper_2504_12471_amd as Pk
    desc = Pk.HeadDesc(2, 3, 8, 4, 1e-6, Pk.F32, 0)
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    scratch = torch.empty(Pk.d2ft_head_scratch_bytes(desc), dtype=torch.uint8, device="cuda")
    with pytest.raises(Pk.D2ftError):
        Pk.d2ft_classifier_fwd_bwd(desc, z(2, 3, 8), z(8), z(8), z(4, 8), z(4), [0, 4], z(2, 3, 8), None, None, None, None, scratch)
    assert Pk.d2ft_embed_scratch_bytes(Pk.EmbedDesc(1, 3, 20, 16, 8, 16, Pk.F32, 0)) == 0     # 20 is not a multiple of 8
    assert Pk.d2ft_embed_scratch_bytes(Pk.EmbedDesc(1, 3, 16, 16, 4, 16, Pk.F32, 0)) == 0     # patch below 8
