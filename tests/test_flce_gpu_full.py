"""Parity at the benchmark's full sizes, in the launch configuration bench.py
times (default logits budget).  The oracle cannot redo 1e13 fp64 flops inside a
GPU test, so it was run once IN FULL by tests/golden/make_golden.py (CPU oracle
only) and the files keep: the loss; exact dX rows and dW rows that cover every
256-row tile of both products, both sides of every possible chunk edge, hot and
never-hit vocabulary ids; the sum and the norm of every 256 x 256 block of dX
and dW; and, for every single row of dX and dW, its norm and its dot product
with a fixed +-1 vector.  Every output element therefore enters at least three
comparisons with oracle values."""
import math
import os

import numpy as np
import pytest
import torch

import workloads
from flce_testlib import TOL, assert_loss, to_host, upload

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TILE = 256

# Noise model behind the bounds on sums and norms (the element-by-element bar is the stated
# one, 2e-2 of max|ref|).  A gradient element is a sum of terms g * x whose factor g, a
# dlogit, comes from a logit that was stored in bf16: the workloads' logits are N(0, 1.3^2),
# below 8 in magnitude, so their absolute rounding error is at most 2^-6, which is the
# RELATIVE error of exp(z) and hence of the softmax term; g itself and the output are rounded
# to bf16 once more each (2^-9).  The errors of different terms are independent with a
# standard deviation of about 2^-7 of the term, so a signed sum of outputs is off by about
# 2^-7 times the Euclidean norm of those outputs however many there are (bound: 6 times
# that); a norm that one large term dominates (a vocabulary row that a single token's
# softmax mass reaches) can be off by that term's full 2^-6 + 2 * 2^-9.
REL_SIGMA = 2.0 ** -7
REL_NORM = 2.0 ** -6 + 2.0 ** -8


def assert_rows_close(name, got, q, scale, rel_to_max, ref_max):
    """got [n, H] against int16-coded oracle rows (value = q * scale, error <= scale / 2):
    max-abs error <= rel_to_max * ref_max with the coding error taken off the bound."""
    ref = q.astype(np.float64) * scale[:, None]
    assert got.shape == ref.shape and np.isfinite(got).all(), name
    err = np.abs(got - ref).max(axis=1)
    coding = np.where((q != 0).any(axis=1), 0.5 * scale, 0.0)   # an all-zero row is stored exactly
    bound = rel_to_max * ref_max - coding
    assert (bound > 0).all()
    worst = int(np.argmax(err / bound))
    assert (err <= bound).all(), \
        f"{name}: sampled row #{worst}: max-abs error {err[worst]:.3e} > {bound[worst]:.3e}"
    return float(err.max() / ref_max)


def assert_whole_matrix(name, M, ref, prefix, signs):
    """Every element of the GPU matrix M [R, C] against the oracle's block sums, block
    norms, row norms and row projections."""
    R, C = M.shape
    Md = M.double()
    assert torch.isfinite(Md).all(), f"{name}: non-finite values"
    nr, nc = (R + TILE - 1) // TILE, (C + TILE - 1) // TILE
    pad = torch.zeros(nr * TILE, nc * TILE, dtype=torch.float64, device=M.device)
    pad[:R, :C] = Md
    blocks = pad.view(nr, TILE, nc, TILE)
    bsum = blocks.sum(dim=(1, 3)).cpu().numpy()
    bsq = blocks.pow(2).sum(dim=(1, 3)).cpu().numpy()
    del pad, blocks
    rsum, rsq = ref[f"{prefix}_blk_sum"], ref[f"{prefix}_blk_sq"]
    assert bsum.shape == rsum.shape
    rnorm = np.sqrt(rsq)
    tiny = 1e-30
    a = np.abs(bsum - rsum) / (6.0 * REL_SIGMA * rnorm + tiny)
    b = np.abs(np.sqrt(bsq) - rnorm) / (REL_NORM * rnorm + tiny)
    assert a.max() <= 1.0, f"{name}: block {np.unravel_index(a.argmax(), a.shape)} sum off by {a.max():.2f} x bound"
    assert b.max() <= 1.0, f"{name}: block {np.unravel_index(b.argmax(), b.shape)} norm off by {b.max():.2f} x bound"
    sg = torch.from_numpy(signs.astype(np.float64)).to(M.device)
    proj = (Md @ sg).cpu().numpy()
    norm = Md.pow(2).sum(dim=1).sqrt().cpu().numpy()
    rproj, rn = ref[f"{prefix}_proj"], ref[f"{prefix}_norm"]
    c = np.abs(proj - rproj) / (6.0 * REL_SIGMA * rn + tiny)
    d = np.abs(norm - rn) / (REL_NORM * rn + tiny)
    assert c.max() <= 1.0, f"{name}: row {c.argmax()} projection off by {c.max():.2f} x bound"
    assert d.max() <= 1.0, f"{name}: row {d.argmax()} norm off by {d.max():.2f} x bound"
    assert (norm[rn == 0.0] == 0.0).all(), f"{name}: a row that is exactly zero in the oracle is not"
    return float(a.max()), float(b.max()), float(c.max()), float(d.max())


def assert_sample_covers_every_tile(rows, vocab, targets, ignore_index, BT, V):
    """The stored sample has a dX row in every 256-row tile of the batch, the rows on both
    sides of every multiple of 256 in the list of rows that have a target (chunk edges of the
    row compaction, whatever the chunk size), and a dW row in every 256-row tile of the
    vocabulary."""
    assert set((rows // TILE).tolist()) == set(range((BT + TILE - 1) // TILE))
    assert set((vocab // TILE).tolist()) == set(range((V + TILE - 1) // TILE))
    val = np.nonzero(targets != ignore_index)[0]
    have = set(rows.tolist())
    for k in range(TILE, len(val), TILE):
        assert int(val[k - 1]) in have and int(val[k]) in have


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_full_size_config_against_stored_oracle(idx):
    _run_full_size(idx)


def test_full_size_several_chunks_at_the_headline_shape():
    # The default plan runs the Llama-3 head as one chunk; a 1 GiB budget taken literally cuts
    # it into two chunks of 4096 rows: fp32 dW partial sums across chunks, chunk edges in dX.
    import paper_2410_10989_amd as flce
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(1 << 30)
        assert flce.flce_num_chunks(8192, 4096, 128256, flce.FLCE_BF16) == 2
        _run_full_size(3)
    finally:
        flce.flce_set_logits_budget_bytes(old)


def test_full_size_without_row_compaction():
    # every row projected (the paper's way), Qwen2 shape: four chunks, dX cut along K
    import paper_2410_10989_amd as flce
    try:
        flce.flce_set_row_compaction(False)
        _run_full_size(4)
    finally:
        flce.flce_set_row_compaction(True)


def _run_full_size(idx):
    import paper_2410_10989_amd as flce
    name = workloads.CONFIGS[idx - 1]["name"]
    ref = np.load(os.path.join(GOLDEN, f"config{idx}_{name}.npz"))
    print(f"case config{idx} {name}: generating inputs", flush=True)
    w = workloads.make_config(idx)
    assert workloads.checksum(w) == str(ref["checksum"]), "input generator drifted from the stored reference"
    assert tuple(ref["shape"]) == (w.BT, w.H, w.V) and int(ref["n_valid"]) == w.n_valid
    assert_sample_covers_every_tile(ref["rows"], ref["vocab"], w.targets, w.ignore_index, w.BT, w.V)
    code = flce.FLCE_BF16
    print(f"  chunks={flce.flce_num_chunks(w.BT, w.H, w.V, code)} x {flce.flce_chunk_rows(w.BT, w.H, w.V, code)} rows, "
          f"workspace {flce.flce_workspace_bytes(w.BT, w.H, w.V, code) / 2**20:.0f} MiB, "
          f"{len(ref['rows'])} dX rows and {len(ref['vocab'])} dW rows sampled", flush=True)
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
    ex = assert_rows_close("dX[sampled rows]", to_host(dX[rows]), ref["dX_q"], ref["dX_scale"], rg,
                           float(ref["dX_absmax"]))
    ew = assert_rows_close("dW[sampled vocab]", to_host(dW[vocab]), ref["dW_q"], ref["dW_scale"], rg,
                           float(ref["dW_absmax"]))
    print(f"  loss {loss.item():.6f} vs {float(ref['loss']):.6f}; dX err {ex:.2e}, dW err {ew:.2e} of max|ref|",
          flush=True)
    signs = ref["signs"]
    sx = assert_whole_matrix("dX", dX, ref, "dX", signs)
    sw = assert_whole_matrix("dW", dW, ref, "dW", signs)
    print("  worst (block sum, block norm, row projection, row norm) as a share of the bound: "
          f"dX {tuple(round(v, 3) for v in sx)}, dW {tuple(round(v, 3) for v in sw)}", flush=True)

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
    # Two DIFFERENT heads on the hidden states of config 3: head 1 has a weight of its own and
    # looks one position further on inside 2048-token sequences (other targets, other ignored
    # rows, other chunk edges), loss weights 1 and 0.8.  dX is the sum over the heads.
    import paper_2410_10989_amd as flce
    from flce_testlib import to_device
    name = workloads.CONFIGS[2]["name"]
    ref = np.load(os.path.join(GOLDEN, f"multihead2_config3_{name}.npz"))
    c = workloads.CONFIGS[2]
    m = workloads.make_multihead(2, c["BT"], c["H"], c["V"], int(ref["seq"]), c["dtype"], c["targets"],
                                 c["ignore"], seed=workloads.BASE_SEED + 3)
    w = m.base
    assert workloads.checksum(w) == str(ref["checksum"])
    assert int(m.targets[1].sum()) == int(ref["t1_sum"])
    assert abs(float(m.Ws[1].astype(np.float64).sum()) - float(ref["w1_sum"])) <= 1e-9 * abs(float(ref["w1_sum"])) + 1e-12
    X = to_device(w.X, "bf16")
    Ws = [to_device(Wj, "bf16") for Wj in m.Ws]
    ts = [torch.from_numpy(tj).cuda() for tj in m.targets]
    nan = float("nan")
    dX = torch.full_like(X, nan)
    dWs = [torch.full_like(Ws[0], nan), torch.full_like(Ws[0], nan)]
    wts = [float(v) for v in ref["weights"]]
    loss, hl, _, _ = flce.flce_multihead_fwd_bwd(X, Ws, ts, wts, w.ignore_index, dX=dX, dWs=dWs)
    torch.cuda.synchronize()
    rl, rg = TOL["bf16"]
    assert_loss(float(loss.item()), float(ref["loss"]), rl)
    for got, want in zip(hl.tolist(), ref["head_losses"].tolist()):
        assert_loss(got, want, rl)
    signs = ref["signs"]
    rows = torch.from_numpy(ref["rows"]).cuda()
    assert set((ref["rows"] // TILE).tolist()) == set(range(w.BT // TILE))
    assert_rows_close("dX[sampled rows]", to_host(dX[rows]), ref["dX_q"], ref["dX_scale"], rg,
                      float(ref["dX_absmax"]))
    print("  dX", assert_whole_matrix("dX", dX, ref, "dX", signs), flush=True)
    for j, dW in enumerate(dWs):
        vocab = ref[f"vocab{j}"]
        assert set((vocab // TILE).tolist()) == set(range(w.V // TILE))
        assert_rows_close(f"dW{j}[sampled vocab]", to_host(dW[torch.from_numpy(vocab).cuda()]),
                          ref[f"dW{j}_q"], ref[f"dW{j}_scale"], rg, float(ref[f"dW{j}_absmax"]))
        print(f"  dW{j}", assert_whole_matrix(f"dW{j}", dW, ref, f"dW{j}", signs), flush=True)
    both_ignored = (ts[0] == w.ignore_index) & (ts[1] == w.ignore_index)
    assert (dX[both_ignored] == 0).all()


def test_full_size_rmsnorm_against_stored_oracle():
    import paper_2410_10989_amd as flce
    from flce_testlib import assert_close, to_device
    name = workloads.CONFIGS[2]["name"]
    ref = np.load(os.path.join(GOLDEN, f"rmsnorm_config3_{name}.npz"))
    w = workloads.make_config(3)
    assert workloads.checksum(w) == str(ref["checksum"])
    h, gamma = workloads.make_rmsnorm_inputs(w)
    assert abs(h.astype(np.float64).sum() - float(ref["h_sum"])) <= 1e-9 * abs(float(ref["h_sum"]))
    assert abs(float(gamma.sum()) - float(ref["gamma_sum"])) <= 1e-6
    assert_sample_covers_every_tile(ref["rows"], ref["vocab"], w.targets, w.ignore_index, w.BT, w.V)
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
    # dh rows differ in scale by the row factors; the bar is relative to the largest entry of
    # the whole dh
    assert_rows_close("dh[sampled rows]", to_host(dh[rows]), ref["dh_q"], ref["dh_scale"], rg,
                      float(ref["dh_absmax"]))
    assert_rows_close("dW[sampled vocab]", to_host(dW[vocab]), ref["dW_q"], ref["dW_scale"], rg,
                      float(ref["dW_absmax"]))
    assert_close("dgamma", to_host(dg), ref["dgamma"].astype(np.float64), rg)
    signs = ref["signs"]
    print("  dh", assert_whole_matrix("dh", dh, ref, "dh", signs), flush=True)
    print("  dW", assert_whole_matrix("dW", dW, ref, "dW", signs), flush=True)
    assert (dh[t == w.ignore_index] == 0).all()


def test_extra_device_memory_does_not_grow_with_BT():
    # At the Llama-3 head: the library-owned workspace, measured through the driver's free-memory
    # counter around each call (all tensors are allocated before), is what flce_workspace_bytes
    # reports, is allocated by the first call, and serves 4, 8 and 16 chunks of rows unchanged
    # (the full logits would be 4.2, 8.4 and 16.8 GB).  (Up to 12 377 rows this shape runs as
    # one chunk, which takes less memory than the chunked plan.)
    import paper_2410_10989_amd as flce
    H, V = 4096, 128256
    code = flce.FLCE_BF16
    flce.flce_release_workspace()
    W = (torch.randn(V, H, device="cuda") * 0.02).to(torch.bfloat16)
    dW = torch.empty_like(W)
    C = flce.flce_chunk_rows(10 ** 7, H, V, code)
    deltas = []
    for BT in (4 * C, 8 * C, 16 * C):
        assert flce.flce_num_chunks(BT, H, V, code) == BT // C
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
        assert flce.flce_workspace_bytes(BT, H, V, code) == flce.flce_workspace_bytes(4 * C, H, V, code)
        assert flce.flce_workspace_bytes(BT, H, V, code) < flce.flce_full_logits_bytes(4 * C, V, code)
        del X, dX, t, loss
    print("  device memory taken by the three calls:", [d >> 20 for d in deltas], "MiB", flush=True)
    assert abs(deltas[0] - flce.flce_workspace_bytes(4 * C, H, V, code)) <= 64 << 20
    assert deltas[1] == 0 and deltas[2] == 0
    flce.flce_release_workspace()
