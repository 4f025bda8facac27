"""Parity of the multi-head entry point (several decoding heads on shared hidden
states) with the fp64 CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads
from flce_testlib import TOL, assert_close, assert_loss, to_device, to_host
from oracle import flce_oracle as oracle

pytestmark = pytest.mark.gpu


def run_heads(m, flags=0, weights="own"):
    import paper_2410_10989_amd as flce
    w = m.base
    X = to_device(w.X, w.dtype)
    Ws = [to_device(a, w.dtype) for a in m.Ws]
    ts = [torch.from_numpy(t).cuda() for t in m.targets]
    n = len(Ws)
    nan = float("nan")
    dX = torch.full_like(X, nan)
    dWs = [torch.full_like(W, nan) for W in Ws]
    loss = torch.full((), nan, dtype=torch.float32, device="cuda")
    hl = torch.full((n,), nan, dtype=torch.float32, device="cuda")
    wts = m.weights if weights == "own" else weights
    flce.flce_multihead_fwd_bwd(X, Ws, ts, wts, w.ignore_index, loss=loss, head_losses=hl, dX=dX,
                                dWs=dWs, flags=flags)
    torch.cuda.synchronize()
    return float(loss.item()), hl.cpu().numpy().astype(np.float64), dX, dWs


def check_heads(m, flags=0):
    import paper_2410_10989_amd as flce
    w = m.base
    print(f"case {w.name} heads={len(m.Ws)} BT={w.BT} H={w.H} V={w.V} {w.dtype} seed={w.seed} "
          f"flags={flags}", flush=True)
    ref = oracle.flce_multihead(w.X, m.Ws, m.targets, m.weights, w.ignore_index)
    loss, hl, dX, dWs = run_heads(m, flags)
    rl, rg = TOL[w.dtype]
    assert_loss(loss, ref.loss, rl)
    for got, want in zip(hl, ref.head_losses):
        assert_loss(float(got), want, rl)
    if not flags & flce.SKIP_DX:
        assert_close("dX", to_host(dX), ref.dX, rg)
        all_ign = np.all([t == w.ignore_index for t in m.targets], axis=0)
        if all_ign.any():   # rows no head has a target for are exact zeros
            assert (to_host(dX)[all_ign] == 0).all()
    else:
        assert torch.isnan(dX.float()).all()   # untouched
    if not flags & flce.SKIP_DW:
        for j, (got, want) in enumerate(zip(dWs, ref.dWs)):
            assert_close(f"dW[{j}]", to_host(got), want, rg)
    else:
        assert all(torch.isnan(d.float()).all() for d in dWs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,BT,H,V,seq", [
    (3, 768, 320, 1344, 128),    # tuned kernels, one chunk, ragged tile edges
    (3, 300, 136, 1000, 50),     # guarded kernels, ragged everywhere
    (5, 256, 64, 512, 64),       # five heads
    (2, 512, 512, 8192, 256),    # long vocabulary, few dX tiles: K-split dX with add
])
def test_heads_match_oracle(dtype, n, BT, H, V, seq):
    m = workloads.make_multihead(n, BT, H, V, seq, dtype, ignore=("iid", 0.1), seed=77 + BT + V)
    check_heads(m)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_heads_with_several_chunks(dtype):
    import paper_2410_10989_amd as flce
    m = workloads.make_multihead(3, 513, 192, 1536, 64, dtype, ignore=("iid", 0.15), seed=991)
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(256 * 1536 * (2 if dtype == "bf16" else 4))
        code = flce.FLCE_BF16 if dtype == "bf16" else flce.FLCE_F32
        assert flce.flce_num_chunks(513, 192, 1536, code) == 3
        check_heads(m)
    finally:
        flce.flce_set_logits_budget_bytes(old)


@pytest.mark.parametrize("flag", ["SKIP_DX", "SKIP_DW"])
def test_frozen_backbone_or_frozen_heads(flag):
    # training only the extra heads needs no dX; the reverse needs no dW
    import paper_2410_10989_amd as flce
    m = workloads.make_multihead(3, 512, 256, 2048, 128, "bf16", seed=31)
    check_heads(m, getattr(flce, flag))


def test_one_head_is_bitwise_the_single_head_call():
    import paper_2410_10989_amd as flce
    from flce_testlib import run_gpu
    m = workloads.make_multihead(1, 768, 320, 1344, 128, "bf16", ignore=("iid", 0.1), seed=5)
    loss1, dX1, dW1 = run_gpu(m.base)
    loss, hl, dX, dWs = run_heads(m, weights=None)
    assert loss == loss1 and hl[0] == loss1
    assert torch.equal(dX.view(torch.int16), dX1.view(torch.int16))
    assert torch.equal(dWs[0].view(torch.int16), dW1.view(torch.int16))


def test_head_without_any_valid_row_contributes_nothing():
    # sequences of 2 tokens: head 2 looks past the end of every sequence
    m = workloads.make_multihead(3, 256, 64, 512, 2, "bf16", seed=8)
    assert (m.targets[2] == m.base.ignore_index).all()
    loss, hl, dX, dWs = run_heads(m)
    assert hl[2] == 0.0 and (to_host(dWs[2]) == 0).all()
    ref = oracle.flce_multihead(m.base.X, m.Ws[:2], m.targets[:2], m.weights[:2], m.base.ignore_index)
    assert_loss(loss, ref.loss, TOL["bf16"][0])
    assert_close("dX", to_host(dX), ref.dX, TOL["bf16"][1])


def test_weights_scale_each_head():
    # weight 0 on head 1: its dW is zero, dX and loss are head 0's alone
    m = workloads.make_multihead(2, 384, 128, 1024, 64, "f32", seed=12)
    loss, hl, dX, dWs = run_heads(m, weights=[1.0, 0.0])
    ref0 = oracle.flce(m.base.X, m.Ws[0], m.targets[0], m.base.ignore_index)
    ref1 = oracle.flce(m.base.X, m.Ws[1], m.targets[1], m.base.ignore_index, want_dX=False,
                       want_dW=False)
    assert_loss(loss, ref0.loss, TOL["f32"][0])
    assert_loss(float(hl[1]), ref1.loss, TOL["f32"][0])    # reported unweighted
    assert (to_host(dWs[1]) == 0).all()
    assert_close("dX", to_host(dX), ref0.dX, TOL["f32"][1])
    assert_close("dW[0]", to_host(dWs[0]), ref0.dW, TOL["f32"][1])
