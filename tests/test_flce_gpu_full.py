"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times (default logits budget).  The oracle cannot redo 1e13 fp64 flops inside a
GPU test, so it was run once by tests/golden/make_golden.py (CPU oracle only)
and its loss, exact dX rows and exact dW rows for a fixed sample are stored;
properties that hold at any size cover the rest of the output."""
import math
import os

import numpy as np
import pytest
import torch

import workloads
from flce_testlib import TOL, assert_close, assert_loss, to_host, upload

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_full_size_config_against_stored_oracle(idx):
    _run_full_size(idx)


def test_full_size_single_chunk_above_2gib():
    # One chunk of 8192 rows: the 2.1 GB dlogits buffer is read K-major by the dW
    # product, whose 32-bit tile offsets then need the descriptor moved mid-way.
    import paper_2410_10989_amd as flce
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(2304 << 20)
        assert flce.flce_num_chunks(8192, 4096, 128256, flce.FLCE_BF16) == 1
        _run_full_size(3)
    finally:
        flce.flce_set_logits_budget_bytes(old)


def _run_full_size(idx):
    import paper_2410_10989_amd as flce
    name = workloads.CONFIGS[idx - 1]["name"]
    ref = np.load(os.path.join(GOLDEN, f"config{idx}_{name}.npz"))
    print(f"case config{idx} {name}: generating inputs", flush=True)
    w = workloads.make_config(idx)
    assert workloads.checksum(w) == str(ref["checksum"]), "input generator drifted from the stored reference"
    assert tuple(ref["shape"]) == (w.BT, w.H, w.V) and int(ref["n_valid"]) == w.n_valid
    code = flce.FLCE_BF16
    print(f"  chunks={flce.flce_num_chunks(w.BT, w.H, w.V, code)} x {flce.flce_chunk_rows(w.BT, w.H, w.V, code)} rows, "
          f"workspace {flce.flce_workspace_bytes(w.BT, w.H, w.V, code) / 2**20:.0f} MiB", flush=True)
    X, W, t = upload(w)
    dX = torch.full_like(X, float("nan"))
    dW = torch.full_like(W, float("nan"))
    loss = torch.full((), float("nan"), dtype=torch.float32, device="cuda")
    flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=dX, dW=dW)
    torch.cuda.synchronize()
    rl, rg = TOL["bf16"]
    assert_loss(float(loss.item()), float(ref["loss"]), rl)

    rows = torch.from_numpy(ref["rows"]).cuda()
    vocab = torch.from_numpy(ref["vocab"]).cuda()
    ex = assert_close("dX[sampled rows]", to_host(dX[rows]), ref["dX_rows"].astype(np.float64), rg)
    ew = assert_close("dW[sampled vocab]", to_host(dW[vocab]), ref["dW_rows"].astype(np.float64), rg)
    print(f"  loss {loss.item():.6f} vs {float(ref['loss']):.6f}; dX err {ex:.2e}, dW err {ew:.2e} of max|ref|",
          flush=True)

    # properties at full scale
    assert torch.isfinite(dX).all() and torch.isfinite(dW).all()
    ign = (t == w.ignore_index)
    assert (dX[ign] == 0).all(), "rows with an ignored target must have zero dX"
    dWd = dW.double()
    # rows of dlogits sum to 0  =>  sum_v dW[v,:] = 0, up to the bf16 rounding of the V stored
    # elements of each column (error std of one element <= 2^-8.8 of its magnitude)
    colsum = dWd.sum(dim=0).abs()
    noise = 6.0 * 2.0 ** -8.8 * dWd.pow(2).sum(dim=0).sqrt()
    worst = (colsum / noise).max().item()
    assert worst <= 1.0, f"sum_v dW[v,:] is {worst:.2f} x the rounding-noise bound"
    never = torch.ones(w.V, dtype=torch.bool, device="cuda")
    never[t[~ign]] = False
    # a class that is never a target only receives positive softmax mass times X: tiny but non-zero
    assert dWd[never].abs().max().item() < dWd[~never].abs().max().item()
    del dWd


def test_budget_change_leaves_headline_result_within_tolerance():
    # Chunk-size invariance on a mid-size shape: 1, 2 and 4 chunks agree with
    # each other far inside the parity bar (the oracle comparison is above).
    import paper_2410_10989_amd as flce
    w = workloads.make(2048, 512, 8192, "bf16", targets="zipf", ignore=("iid", 0.1), seed=321)
    X, W, t = upload(w)
    old = flce.flce_get_logits_budget_bytes()
    outs = []
    try:
        for rows in (2048, 1024, 512):
            flce.flce_set_logits_budget_bytes(rows * 8192 * 2)
            assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16) == 2048 // rows
            loss, dX, dW = flce.flce_fwd_bwd(X, W, t, w.ignore_index)
            torch.cuda.synchronize()
            outs.append((loss.item(), dX.float(), dW.float()))
    finally:
        flce.flce_set_logits_budget_bytes(old)
    for o in outs[1:]:
        assert abs(o[0] - outs[0][0]) <= 1e-6 * abs(outs[0][0])
        assert torch.equal(o[1], outs[0][1])          # dX rows never mix chunks
        assert (o[2] - outs[0][2]).abs().max().item() <= 1e-2 * outs[0][2].abs().max().item()


def test_full_size_two_heads_against_stored_oracle():
    # Two heads with the SAME weight and targets and loss weights 0.75 / 0.25: by linearity the
    # loss and dX are the single-head ones and dW_j is weight_j times the single-head dW, so the
    # stored config-3 reference covers the multi-head entry point at full size (dX summed over
    # heads through the bf16 addend of the dX product, per-head scaling of the gradients).
    import paper_2410_10989_amd as flce
    name = workloads.CONFIGS[2]["name"]
    ref = np.load(os.path.join(GOLDEN, f"config3_{name}.npz"))
    w = workloads.make_config(3)
    assert workloads.checksum(w) == str(ref["checksum"])
    X, W, t = upload(w)
    nan = float("nan")
    dX = torch.full_like(X, nan)
    dWs = [torch.full_like(W, nan), torch.full_like(W, nan)]
    wts = [0.75, 0.25]
    loss, hl, _, _ = flce.flce_multihead_fwd_bwd(X, [W, W], [t, t], wts, w.ignore_index, dX=dX, dWs=dWs)
    torch.cuda.synchronize()
    rl, rg = TOL["bf16"]
    assert_loss(float(loss.item()), float(ref["loss"]), rl)
    for v in hl.tolist():
        assert_loss(v, float(ref["loss"]), rl)
    rows = torch.from_numpy(ref["rows"]).cuda()
    vocab = torch.from_numpy(ref["vocab"]).cuda()
    assert_close("dX[sampled rows]", to_host(dX[rows]), ref["dX_rows"].astype(np.float64), rg)
    for wt, dW in zip(wts, dWs):
        assert_close("dW[sampled vocab]", to_host(dW[vocab]), wt * ref["dW_rows"].astype(np.float64), rg)
    assert torch.isfinite(dX).all() and all(torch.isfinite(d).all() for d in dWs)
    assert (dX[t == w.ignore_index] == 0).all()


def test_full_size_rmsnorm_against_stored_oracle():
    import paper_2410_10989_amd as flce
    from flce_testlib import to_device
    name = workloads.CONFIGS[2]["name"]
    ref = np.load(os.path.join(GOLDEN, f"rmsnorm_config3_{name}.npz"))
    w = workloads.make_config(3)
    assert workloads.checksum(w) == str(ref["checksum"])
    h, gamma = workloads.make_rmsnorm_inputs(w)
    assert abs(h.astype(np.float64).sum() - float(ref["h_sum"])) <= 1e-9 * abs(float(ref["h_sum"]))
    assert abs(float(gamma.sum()) - float(ref["gamma_sum"])) <= 1e-6
    hd, gd, Wd = to_device(h, "bf16"), to_device(gamma, "bf16"), to_device(w.W, "bf16")
    t = torch.from_numpy(w.targets).cuda()
    nan = float("nan")
    dh, dg, dW = torch.full_like(hd, nan), torch.full_like(gd, nan), torch.full_like(Wd, nan)
    loss = torch.full((), nan, dtype=torch.float32, device="cuda")
    flce.flce_rmsnorm_fwd_bwd(hd, gd, float(ref["eps"]), Wd, t, w.ignore_index, loss=loss, dh=dh,
                              dgamma=dg, dW=dW)
    torch.cuda.synchronize()
    rl, rg = TOL["bf16"]
    assert_loss(float(loss.item()), float(ref["loss"]), rl)
    rows = torch.from_numpy(ref["rows"]).cuda()
    vocab = torch.from_numpy(ref["vocab"]).cuda()
    # dh rows differ in scale by the row factors, so the bar is relative to the largest entry of
    # the whole dh, which the reference stores
    assert_close("dh[sampled rows]", to_host(dh[rows]), ref["dh_rows"].astype(np.float64), rg,
                 ref_max=float(ref["dh_absmax"]))
    assert_close("dW[sampled vocab]", to_host(dW[vocab]), ref["dW_rows"].astype(np.float64), rg)
    assert_close("dgamma", to_host(dg), ref["dgamma"].astype(np.float64), rg)
    assert torch.isfinite(dh).all() and torch.isfinite(dW).all()
    assert (dh[t == w.ignore_index] == 0).all()


def test_extra_device_memory_does_not_grow_with_BT():
    # At the Llama-3 head: the library-owned workspace, measured through the driver's free-memory
    # counter around each call (all tensors are allocated before), is what flce_workspace_bytes
    # reports, is allocated by the first call, and serves 2, 4 and 8 chunks of rows unchanged
    # (the full logits would be 2.1, 4.2 and 8.4 GB).
    import paper_2410_10989_amd as flce
    H, V = 4096, 128256
    code = flce.FLCE_BF16
    flce.flce_release_workspace()
    W = (torch.randn(V, H, device="cuda") * 0.02).to(torch.bfloat16)
    dW = torch.empty_like(W)
    C = flce.flce_chunk_rows(10 ** 7, H, V, code)
    deltas = []
    for BT in (2 * C, 4 * C, 8 * C):
        g = torch.Generator(device="cuda").manual_seed(BT)
        X = torch.randn(BT, H, device="cuda", generator=g).to(torch.bfloat16)
        t = torch.randint(0, V, (BT,), device="cuda", generator=g)
        dX = torch.empty_like(X)
        loss = torch.empty((), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        flce.flce_fwd_bwd(X, W, t, loss=loss, dX=dX, dW=dW)
        torch.cuda.synchronize()
        deltas.append(free_before - torch.cuda.mem_get_info()[0])
        assert math.isfinite(loss.item()) and abs(loss.item() - math.log(V)) < 1.0
        assert flce.flce_workspace_bytes(BT, H, V, code) == flce.flce_workspace_bytes(2 * C, H, V, code)
        assert flce.flce_workspace_bytes(BT, H, V, code) < flce.flce_full_logits_bytes(8 * C, V, code)
        del X, dX, t, loss
    print("  device memory taken by the three calls:", [d >> 20 for d in deltas], "MiB", flush=True)
    assert abs(deltas[0] - flce.flce_workspace_bytes(2 * C, H, V, code)) <= 64 << 20
    assert deltas[1] == 0 and deltas[2] == 0
    flce.flce_release_workspace()
