"""One whole fine-tune step on the GPU - patch embedding, a stack of blocks with op codes, classifier + loss,
backward through everything - against the same composition of the oracle's pieces (Sec. IV-A's 2 + L*H subnets)."""
import numpy as np
import pytest

import d2ft_inputs as di
from helpers import FLAG_GATE_FFN, rel_inf

pytestmark = pytest.mark.gpu

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP


@pytest.mark.parametrize("dtype,gate", [("f32", False), ("bf16", True)])
def test_full_step(dtype, gate):
    import torch
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    rng = np.random.default_rng(131)
    B, C, Himg, Wimg, Pp, D, H, Dm, L, n_cls = 4, 3, 32, 32, 8, 128, 2, 256, 2, 10
    T = 1 + (Himg // Pp) * (Wimg // Pp)
    w = di.Workload("full_step", B, T, D, H, 64, Dm, L, dtype)
    grid = (lambda a: di.round_to_bf16(np.asarray(a, np.float32))) if dtype == "bf16" else (lambda a: np.asarray(a, np.float32))
    emb = dict(images=grid(rng.standard_normal((B, C, Himg, Wimg))), w_pe=grid(rng.standard_normal((D, C * Pp * Pp)) * 0.05),
               b_pe=grid(rng.standard_normal(D) * 0.1), cls=grid(rng.standard_normal(D)), pos=grid(rng.standard_normal((T, D)) * 0.5))
    blocks = [di.draw_block_weights(rng, w) for _ in range(L)]
    head = dict(ln_g=grid(1 + 0.1 * rng.standard_normal(D)), ln_b=grid(0.1 * rng.standard_normal(D)),
                w_c=grid(rng.standard_normal((n_cls, D)) * 0.2), b_c=grid(rng.standard_normal(n_cls) * 0.1))
    labels = rng.integers(0, n_cls, size=B)
    ops = np.array([[FULL, FWD], [SKIP, FULL]], dtype=np.uint8)

    # ---- oracle ----
    tok, ecache = orc.patch_embed_fwd(emb["images"], emb["w_pe"], emb["b_pe"], emb["cls"], emb["pos"], Pp)
    y, caches = orc.stack_fwd(blocks, ops, tok, 64, gate_ffn=gate)
    rloss, _, hcache = orc.classifier_fwd(y, head["ln_g"], head["ln_b"], head["w_c"], head["b_c"], labels)
    dy, rgh = orc.classifier_bwd(hcache)
    dtok, rgb = orc.stack_bwd(blocks, caches, dy)
    rge = orc.patch_embed_bwd(ecache, dtok)

    # ---- GPU ----
    code = P.BF16 if dtype == "bf16" else P.F32
    edesc = P.EmbedDesc(B, C, Himg, Wimg, Pp, D, code, 0)
    hdesc = P.HeadDesc(B, T, D, n_cls, 1e-6, code, 0)
    bdesc = P.make_desc(B, T, D, H, Dm, dtype, flags=FLAG_GATE_FFN if gate else 0)
    dev = lambda a: P.to_device(a, dtype)
    de = {k: dev(v) for k, v in emb.items()}
    dh = {k: dev(v) for k, v in head.items()}
    tokens = torch.empty((B, T, D), dtype=P.torch_dtype(dtype), device="cuda")
    esaved = torch.empty(P.d2ft_embed_saved_bytes(edesc), dtype=torch.uint8, device="cuda")
    escr = torch.empty(P.d2ft_embed_scratch_bytes(edesc), dtype=torch.uint8, device="cuda")
    P.d2ft_patch_embed_fwd(edesc, de["images"], de["w_pe"], de["b_pe"], de["cls"], de["pos"], tokens, esaved, escr)
    stack = P.BlockStack(bdesc, [{k: dev(v) for k, v in bw.items()} for bw in blocks], dtype, grad_fields=list(P.WEIGHT_FIELDS))
    yd = stack.forward(tokens, ops)
    dyd = torch.empty_like(yd)
    gh = {k: torch.empty_like(v) for k, v in dh.items()}
    hscr = torch.empty(P.d2ft_head_scratch_bytes(hdesc), dtype=torch.uint8, device="cuda")
    loss = P.d2ft_classifier_fwd_bwd(hdesc, yd, dh["ln_g"], dh["ln_b"], dh["w_c"], dh["b_c"], labels, dyd, gh["ln_g"], gh["ln_b"],
                                     gh["w_c"], gh["b_c"], hscr)
    dtokd = stack.backward(dyd, ops)
    ge = {k: torch.empty_like(de[k]) for k in ("w_pe", "b_pe", "cls", "pos")}
    P.d2ft_patch_embed_bwd(edesc, dtokd, ge["w_pe"], ge["b_pe"], ge["cls"], ge["pos"], esaved, escr)
    torch.cuda.synchronize()

    tol = 1e-4 if dtype == "f32" else 2e-2
    assert abs(loss - rloss) <= tol * max(1.0, abs(rloss)), (loss, rloss)
    errs = {"dtokens": rel_inf(dtokd.float().cpu().numpy(), dtok)}
    for k in ge:
        errs["embed." + k] = rel_inf(ge[k].float().cpu().numpy(), rge[k])
    for k in gh:
        errs["head." + k] = rel_inf(gh[k].float().cpu().numpy(), rgh[k])
    for l in range(L):
        for k in ("w_qkv", "w_o", "w1", "w2"):
            errs[f"block{l}.{k}"] = rel_inf(stack.grads[l][k].float().cpu().numpy(), rgb[l][k])
    print(f"[full step {dtype} gate={gate}] loss={loss:.5f} ref={rloss:.5f} max err {max(errs.values()):.2e}", flush=True)
    assert all(v <= tol for v in errs.values()), errs
    # block 1, head 0 is a shortcut subnet: exact zeros
    g = stack.grads[1]["w_qkv"].float().cpu().numpy()
    assert np.all(g[:, 0] == 0.0)
