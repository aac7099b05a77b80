"""GPU parity of the token embedding and the language-modelling head + loss (Section 4.3: first and last pipeline
stage) against the oracle, through the C ABI.

Embedding forward is a copy: bit-exact.  Embedding backward sums bf16 / fp32 rows in fp32: 1e-6.  Head: fp32 within
1e-4, bf16 within 2e-2, max|gpu - oracle| / max|oracle| per output tensor; the scalar loss to the same relative
bound.
"""
import numpy as np
import pytest
import torch

import swarm_synth as synth
from oracle import head as oh
from stage_util import max_norm_err

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _dev(a, wl):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(torch.bfloat16) if wl.dtype == "bf16" else t).cuda()


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def check_embedding(wl):
    import paper_2301_11913_amd as sw
    table, _ = synth.make_head_params(wl)
    tokens, _, _, dxe = synth.make_head_inputs(wl)
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    tok_d, tab_d = torch.from_numpy(tokens).cuda(), _dev(table, wl)
    x = torch.full((wl.tokens, wl.d_model), 7.0, dtype=dt, device="cuda")
    sw.swarm_embedding_forward(tok_d, tab_d, wl.vocab, x)
    grad = torch.full((wl.vocab_rows, wl.d_model), 0.5, dtype=torch.float32, device="cuda")    # += into a non-zero buffer
    sw.swarm_embedding_backward(tok_d, _dev(dxe, wl), wl.vocab, grad)
    again = torch.full_like(grad, 0.5)
    sw.swarm_embedding_backward(tok_d, _dev(dxe, wl), wl.vocab, again)
    torch.cuda.synchronize()
    assert np.array_equal(_f64(x), oh.embedding_forward(tokens, table))
    ref = np.full((wl.vocab_rows, wl.d_model), 0.5)
    oh.embedding_backward(tokens, dxe, ref)
    assert max_norm_err(_f64(grad), ref) <= 1e-6
    assert torch.equal(grad, again)                                                        # reproducible
    untouched = np.ones(wl.vocab_rows, dtype=bool)
    untouched[np.unique(tokens)] = False
    assert np.all(_f64(grad)[untouched] == 0.5)                                           # rows of absent ids: untouched


def check_head(wl, dt=np.float64, evaluate=True):
    import paper_2301_11913_amd as sw
    _, head = synth.make_head_params(wl)
    _, targets, x, _ = synth.make_head_inputs(wl)
    cfg = sw.HeadConfig(wl.d_model, wl.vocab, wl.vocab_rows, wl.tokens, wl.dtype, wl.ln_eps)
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    hp = {k: _dev(v, wl) for k, v in head.items()}
    gp = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in head.items()}
    ws = torch.empty(sw.swarm_head_workspace_bytes(cfg, True), dtype=torch.uint8, device="cuda")
    loss = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    tok = torch.full((wl.tokens,), -1.0, dtype=torch.float32, device="cuda")
    dx = torch.full((wl.tokens, wl.d_model), 7.0, dtype=tdt, device="cuda")
    xd, td = _dev(x, wl), torch.from_numpy(targets).cuda()
    sw.swarm_head_loss_backward(cfg, hp, xd, td, loss, tok, dx, gp, ws)
    torch.cuda.synchronize()
    grads = {k: np.zeros(v.shape, dtype=dt) for k, v in head.items()}
    rl, rtok, rdx = oh.head_loss_backward(x, targets, head, wl.vocab, grads, wl.ln_eps, dt)
    tol = TOL[wl.dtype]
    errs = {"loss": abs(loss.item() - rl) / abs(rl), "token_loss": max_norm_err(_f64(tok), rtok),
            "dx": max_norm_err(_f64(dx), rdx)}
    for k in grads:
        errs[k] = max_norm_err(_f64(gp[k]), grads[k])
    print(wl.name, wl.dtype, "loss %.4f" % rl, {k: "%.2e" % v for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if not (v <= tol)}
    assert not bad, bad
    assert np.all(_f64(gp["w_vocab"])[wl.vocab:] == 0.0)          # padding rows: zero gradient
    if evaluate:                                                   # the loss-only entry point gives the same numbers
        loss2 = torch.zeros(1, dtype=torch.float32, device="cuda")
        tok2 = torch.zeros(wl.tokens, dtype=torch.float32, device="cuda")
        sw.swarm_head_loss(cfg, hp, xd, td, loss2, tok2, ws)
        torch.cuda.synchronize()
        assert torch.equal(loss, loss2) and torch.equal(tok, tok2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,V,rows,T", [
    (64, 11, 16, 37),          # tiny vocabulary: every id repeats many times
    (128, 1000, 1000, 150),
    (256, 5000, 5120, 513),    # ragged token count, padded vocabulary
    (1024, 2000, 2048, 256),
])
def test_embedding(dtype, d, V, rows, T):
    check_embedding(synth.HeadWorkload("emb", dtype, d, V, rows, T, seed=900 + d + V + T))


def test_embedding_all_tokens_equal():
    """T positions, one id: the single first-occurrence workgroup sums every row, in position order."""
    import paper_2301_11913_amd as sw
    wl = synth.HeadWorkload("emb1", "bf16", 256, 50, 64, 700, seed=5)
    _, _, _, dxe = synth.make_head_inputs(wl)
    tokens = np.full(wl.tokens, 17, dtype=np.int32)
    grad = torch.zeros((wl.vocab_rows, wl.d_model), dtype=torch.float32, device="cuda")
    sw.swarm_embedding_backward(torch.from_numpy(tokens).cuda(), _dev(dxe, wl), wl.vocab, grad)
    torch.cuda.synchronize()
    ref = np.zeros((wl.vocab_rows, wl.d_model))
    oh.embedding_backward(tokens, dxe, ref)
    assert max_norm_err(_f64(grad), ref) <= 1e-6
    assert np.count_nonzero(_f64(grad).any(axis=1)) == 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,V,rows,T", [
    (64, 11, 16, 37),
    (128, 1000, 1000, 150),
    (256, 5000, 5120, 513),
    (1024, 2000, 2048, 256),   # MFMA tile shapes
])
def test_head_loss_backward(dtype, d, V, rows, T):
    check_head(synth.HeadWorkload("head", dtype, d, V, rows, T, seed=300 + d + V + T))


def test_head_full_size():
    """The Section 4.3 model's head as bench.py times it: d_model 4096, 50257 tokens padded to 50432 rows, one
    2048-token sequence."""
    check_head(synth.HEAD_WORKLOADS["head_gpt2vocab_bf16_d4096"], dt=np.float32)
    check_embedding(synth.HEAD_WORKLOADS["head_gpt2vocab_bf16_d4096"])
