"""Parity of the HIP path (called through the C ABI) with the fp64 CPU oracle,
element by element, on seeded inputs at sizes the oracle finishes in seconds:
several tiles, ragged tails, several chunks, and the degenerate cases."""
import numpy as np
import pytest
import torch

import workloads
from flce_testlib import TOL, assert_close, assert_loss, run_gpu, to_host, upload
from oracle import flce_oracle as oracle

pytestmark = pytest.mark.gpu


def to_device_like(ref: torch.Tensor, a: np.ndarray) -> torch.Tensor:
    from flce_testlib import to_device
    return to_device(a, "bf16" if ref.dtype == torch.bfloat16 else "f32")


def check_full(w, flags=0):
    import paper_2410_10989_amd as flce
    print(f"case {w.name} BT={w.BT} H={w.H} V={w.V} {w.dtype} seed={w.seed} flags={flags} "
          f"chunks={flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16 if w.dtype == 'bf16' else flce.FLCE_F32)}",
          flush=True)
    ref = oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    loss, dX, dW = run_gpu(w, flags)
    rl, rg = TOL[w.dtype]
    assert_loss(loss, ref.loss, rl)
    if not flags & flce.SKIP_DX:
        assert_close("dX", to_host(dX), ref.dX, rg)
        ign = w.targets == w.ignore_index
        if ign.any():   # ignored rows are exact zeros
            assert (to_host(dX)[ign] == 0).all()
    if not flags & flce.SKIP_DW:
        assert_close("dW", to_host(dW), ref.dW, rg)
    return loss, dX, dW


def test_config1_tiny_fp32():
    check_full(workloads.make_config(1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("BT,H,V,ignore", [
    (300, 136, 1000, ("iid", 0.1)),     # ragged in every dimension, aligned K
    (77, 100, 333, ("iid", 0.3)),       # H not a multiple of the vector width
    (1, 64, 129, ("none",)),            # a single row
    (129, 8, 2, ("iid", 0.2)),          # two classes
    (513, 256, 2048, ("iid", 0.05)),    # tile-aligned except one trailing row
    (640, 72, 4100, ("pad", 128, 60)),  # padding runs
    (768, 320, 1344, ("iid", 0.1)),     # tuned-kernel path: K multiples of 64, ragged tile edges
    (256, 64, 256, ("none",)),          # tuned-kernel path: exactly one macro tile
    (832, 192, 2112, ("iid", 0.5)),     # tuned-kernel path, half the rows ignored
    (520, 256, 3001, ("iid", 0.1)),     # tuned kernels with V % 64 != 0: zero-padded K tail of dX
    (1000, 128, 50257 // 8, ("iid", 0.1)),   # odd V (a GPT-2 style vocabulary, scaled down) and rows % 64 != 0
    (70, 64, 65, ("none",)),            # one column past a K step; fewer rows than a K step
    (640, 1032, 4096, ("iid", 0.1)),    # guarded kernels over many tiles and K steps in every product
    (5, 8, 1, ("none",)),               # one class: the loss and every gradient are exactly zero
    (9, 1, 5, ("iid", 0.2)),            # hidden size one
    (1, 4096, 50257, ("none",)),        # a single row against a full-size head: K = 1 in the dW product
    (3, 2048, 262144 + 7, ("iid", 0.34)),   # three rows, a quarter of a million classes, 1 GB of W in fp32
])
def test_ragged_shapes(dtype, BT, H, V, ignore):
    check_full(workloads.make(BT, H, V, dtype, ignore=ignore, seed=1000 + BT + V, name="ragged"))


def test_dx_is_cut_along_k_when_the_tile_count_leaves_a_poor_last_round():
    # 17 x 16 = 272 output tiles of dX on 256 CUs would run as two rounds; the scheduler
    # cuts K = V in two ranges instead (fp32 partials, fixed-order sum)
    check_full(workloads.make(4352, 4096, 8192, "bf16", ignore=("iid", 0.1), seed=272, name="tail"))


@pytest.mark.parametrize("ignore_frac", [0.0, 0.4, 0.75])
def test_dx_k_ranges_follow_the_live_row_count(ignore_frac):
    # 3 x 1 output tiles of dX, K = V = 16384 (256 K steps): a full chunk is cut into 4 K
    # ranges; with rows ignored the device picks fewer ranges for the live tiles (2 tile rows:
    # 3 ranges, 1 tile row: 4 again), sums their partial results in a fixed order, and the
    # result matches the oracle element by element; without compaction the host's choice runs
    import paper_2410_10989_amd as flce
    assert flce.flce_dx_k_ranges(600, 256, 16384, flce.FLCE_BF16) == 4
    w = workloads.make(600, 256, 16384, "bf16", ignore=("iid", ignore_frac) if ignore_frac else ("none",),
                       seed=4242 + int(100 * ignore_frac), name="k_ranges")
    on = check_full(w)
    try:
        flce.flce_set_row_compaction(False)
        off = check_full(w)
    finally:
        flce.flce_set_row_compaction(True)
    err = (on[1].float() - off[1].float()).abs().max().item()
    assert err <= 2.0 ** -7 * off[1].float().abs().max().item()   # other K ranges: other rounding, not more


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_several_chunks_with_ragged_last_chunk(dtype):
    # A budget of 256 rows of logits forces 3 chunks (256, 256, 1 rows); the
    # result must be the one-chunk result within tolerance and match the oracle.
    import paper_2410_10989_amd as flce
    w = workloads.make(513, 192, 1536, dtype, ignore=("iid", 0.15), seed=4242, name="chunked")
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(256 * 1536 * (4 if dtype == "f32" else 2))
        code = flce.FLCE_F32 if dtype == "f32" else flce.FLCE_BF16
        assert flce.flce_num_chunks(w.BT, w.H, w.V, code) == 3
        check_full(w)
    finally:
        flce.flce_set_logits_budget_bytes(old)


def _random_cases(n, seed):
    import random
    rng = random.Random(seed)
    cases = []
    for k in range(n):
        cases.append((rng.choice(["f32", "bf16"]), rng.choice([1, 7, 64, 130, 257, 600, 1100]),
                      rng.choice([8, 24, 64, 72, 136, 256, 520]),
                      rng.choice([3, 64, 257, 1000, 2048, 5003, 9000]),
                      rng.choice([("none",), ("iid", 0.2), ("iid", 0.7)]), rng.choice([0, 256, 512]), k))
    return cases


@pytest.mark.parametrize("dtype,BT,H,V,ignore,budget_rows,k", _random_cases(32, 20241010))
def test_random_shapes_and_budgets(dtype, BT, H, V, ignore, budget_rows, k):
    # seeded draws over both storage types, ragged and tiny dimensions, few-tile dX
    # products (cut along K) and logits budgets of 256 / 512 rows (several chunks)
    import paper_2410_10989_amd as flce
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(budget_rows * ((V + 63) // 64 * 64) * (4 if dtype == "f32" else 2))
        check_full(workloads.make(BT, H, V, dtype, ignore=ignore, seed=7000 + k, name="random"))
    finally:
        flce.flce_set_logits_budget_bytes(old)


def test_zipf_targets_medium_bf16():
    check_full(workloads.make(1024, 512, 8192, "bf16", targets="zipf", ignore=("iid", 0.05),
                              seed=99, name="zipf"))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_rows_ignored_gives_zeros(dtype):
    w = workloads.make(130, 64, 300, dtype, seed=7, name="all_ignored")
    w.targets[:] = w.ignore_index
    loss, dX, dW = run_gpu(w)
    assert loss == 0.0
    assert (to_host(dX) == 0).all() and (to_host(dW) == 0).all()


def test_skip_flags():
    import paper_2410_10989_amd as flce
    w = workloads.make(260, 128, 700, "bf16", ignore=("iid", 0.1), seed=31, name="skip")
    check_full(w, flce.SKIP_DX)
    check_full(w, flce.SKIP_DW)


def test_runs_are_bitwise_reproducible():
    w = workloads.make(700, 256, 3000, "bf16", ignore=("iid", 0.1), seed=55, name="repro")
    a = run_gpu(w)
    b = run_gpu(w)
    assert a[0] == b[0]
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])


def test_large_logits_do_not_overflow():
    w = workloads.make(64, 128, 512, "f32", seed=8, name="large_logits", x_std=8.0, w_std=2.0)
    ref = oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    loss, dX, dW = run_gpu(w)
    assert_loss(loss, ref.loss, 1e-5)
    assert_close("dX", to_host(dX), ref.dX, 1e-4)
    assert_close("dW", to_host(dW), ref.dW, 1e-4)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("BT,V,pad", [(37, 1000, 0), (16, 4099, 5), (3, 7, 0), (200, 40960, 0),
                                        (70001, 136, 0)])   # the last: more rows than one launch of the row kernel takes
def test_standalone_cross_entropy(dtype, BT, V, pad):
    import paper_2410_10989_amd as flce
    g = np.random.default_rng(BT * 7 + V)
    Z = (g.standard_normal((BT, V)) * 2.0).astype(np.float32)
    if dtype == "bf16":
        workloads.round_to_bf16(Z)
    t = g.integers(0, V, size=BT).astype(np.int64)
    t[::5] = -100
    ref_loss, ref_G, _ = oracle.cross_entropy(Z.astype(np.float64), t, -100)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    buf = torch.zeros((BT, V + pad), dtype=tdt, device="cuda")
    buf[:, :V] = torch.from_numpy(Z).cuda().to(tdt)
    view = buf[:, :V]
    loss = flce.flce_cross_entropy_inplace(view, torch.from_numpy(t).cuda(), -100)
    torch.cuda.synchronize()
    rl, rg = TOL[dtype]
    assert_loss(float(loss.item()), ref_loss, rl)
    assert_close("dZ", to_host(view), ref_G, rg)
    if pad:
        assert (to_host(buf[:, V:]) == 0).all()   # the row padding is not touched


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_chunk_of_more_than_65536_rows(dtype):
    # a small vocabulary makes the automatic budget hold the whole batch: ONE chunk of 150 001 rows,
    # i.e. 586 tile rows in the products, a row kernel launched in three pieces, and (bf16) the
    # row compaction collecting 105 000 rows in one go
    import paper_2410_10989_amd as flce
    w = workloads.make(150001, 64, 200, dtype, ignore=("iid", 0.3), seed=77, name="many_rows")
    assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16 if dtype == "bf16" else flce.FLCE_F32) == 1
    check_full(w)


def test_ragged_vocabulary_with_a_poisoned_workspace():
    # V % 64 != 0: the dX product reads the dlogits rows up to the next multiple of 64; those
    # padding columns must have been set to zero, whatever the lent workspace held before
    import paper_2410_10989_amd as flce
    w = workloads.make(384, 128, 1000, "bf16", ignore=("iid", 0.1), seed=64, name="poisoned_ws")
    need = flce.flce_workspace_bytes(w.BT, w.H, w.V, flce.FLCE_BF16)
    ws = torch.full((need // 2 + 128,), float("nan"), dtype=torch.bfloat16, device="cuda")
    try:
        flce.flce_set_workspace(ws)
        check_full(w)
    finally:
        flce.flce_set_workspace(None)


def test_lent_workspace_that_is_too_small_is_refused():
    import paper_2410_10989_amd as flce
    w = workloads.make(256, 128, 1024, "bf16", seed=3, name="small_ws")
    X, W, t = upload(w)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    try:
        flce.flce_set_workspace(ws)
        with pytest.raises(flce.FlceError) as e:
            flce.flce_fwd_bwd(X, W, t, w.ignore_index)
        assert e.value.status == 5
    finally:
        flce.flce_set_workspace(None)
    check_full(w)   # and the library-owned workspace still works afterwards


def test_call_on_a_side_stream_is_ordered_with_that_stream():
    # the whole call is enqueued on the caller's stream: work queued before it on that stream
    # (here: the upload-side fill of X) is seen, and a stream synchronise is all the caller needs
    import paper_2410_10989_amd as flce
    w = workloads.make(640, 256, 2048, "bf16", ignore=("iid", 0.1), seed=17, name="side_stream")
    ref = oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    Xh, W, t = upload(w)
    side = torch.cuda.Stream()
    X = torch.empty_like(Xh)
    dX, dW = torch.empty_like(Xh), torch.empty_like(W)
    loss = torch.empty((), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        X.copy_(Xh, non_blocking=True)
        flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=dX, dW=dW)   # current stream = side
    side.synchronize()
    rl, rg = TOL["bf16"]
    assert_loss(float(loss.item()), ref.loss, rl)
    assert_close("dX", to_host(dX), ref.dX, rg)
    assert_close("dW", to_host(dW), ref.dW, rg)


def test_call_can_be_captured_in_a_graph_and_replayed():
    # The call is kernel launches on the caller's stream only (no allocation once the workspace
    # exists, no memset, no synchronisation), so it can be recorded into a HIP graph.  Every
    # replay, with the program's own eager work in between, must give the eager result's bits.
    import paper_2410_10989_amd as flce
    w = workloads.make(513, 192, 1536, "bf16", ignore=("iid", 0.1), seed=23, name="graph")
    X0, W, t = upload(w)
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(256 * 1536 * 2)      # 3 chunks: the whole loop is captured
        X = X0.clone()
        loss = torch.empty((), dtype=torch.float32, device="cuda")
        dX, dW = torch.empty_like(X), torch.empty_like(W)
        flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=dX, dW=dW)   # sizes the workspace
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=dX, dW=dW)
        for scale in (1.0, 0.5, -2.0, 1.0):
            X.copy_(X0 * scale)
            dX.fill_(float("nan"))
            dW.fill_(float("nan"))
            loss.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            got = (loss.item(), dX.clone(), dW.clone())
            e_loss, e_dX, e_dW = flce.flce_fwd_bwd(X, W, t, w.ignore_index)   # eager, fresh outputs
            torch.cuda.synchronize()
            assert got[0] == e_loss.item()
            assert torch.equal(got[1].view(torch.int16), e_dX.view(torch.int16))
            assert torch.equal(got[2].view(torch.int16), e_dW.view(torch.int16))
    finally:
        flce.flce_set_logits_budget_bytes(old)


def test_multihead_and_rmsnorm_entries_can_be_captured_too():
    # same property for the other two entry points (dX accumulated over heads; dgamma partial
    # sums cleared by a kernel inside the call): replays equal the eager results bit for bit
    import paper_2410_10989_amd as flce
    m = workloads.make_multihead(2, 513, 192, 1536, 64, "bf16", ignore=("iid", 0.1), seed=29)
    X0, W0, t0 = upload(m.base)
    Ws = [W0] + [to_device_like(W0, m.Ws[1])]
    ts = [torch.from_numpy(t).cuda() for t in m.targets]
    h_np, gamma_np = workloads.make_rmsnorm_inputs(m.base)
    gamma = to_device_like(W0, gamma_np)
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(256 * 1536 * 2)
        X = X0.clone()
        loss, loss_n = (torch.empty((), dtype=torch.float32, device="cuda") for _ in range(2))
        hl = torch.empty(2, dtype=torch.float32, device="cuda")
        dX, dh = torch.empty_like(X), torch.empty_like(X)
        dWs = [torch.empty_like(W0) for _ in range(2)]
        dWn, dgamma = torch.empty_like(W0), torch.empty_like(gamma)

        def heads(loss, hl, dX, dWs):
            return flce.flce_multihead_fwd_bwd(X, Ws, ts, list(m.weights), m.base.ignore_index, loss=loss,
                                               head_losses=hl, dX=dX, dWs=dWs)

        def norm(loss, dh, dgamma, dW):
            return flce.flce_rmsnorm_fwd_bwd(X, gamma, 1e-6, W0, ts[0], m.base.ignore_index, loss=loss,
                                             dh=dh, dgamma=dgamma, dW=dW)

        heads(loss, hl, dX, dWs)            # size the workspaces
        norm(loss_n, dh, dgamma, dWn)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            heads(loss, hl, dX, dWs)
            norm(loss_n, dh, dgamma, dWn)
        for scale in (1.0, -0.5, 1.0):
            X.copy_(X0 * scale)
            for b in (dX, dh, dWn, dgamma, *dWs):
                b.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            got = [x.clone() for x in (loss, hl, dX, *dWs, loss_n, dh, dgamma, dWn)]
            e_hl = torch.empty_like(hl)
            e = heads(torch.empty_like(loss), e_hl, torch.empty_like(dX), [torch.empty_like(W0) for _ in range(2)])
            n = norm(torch.empty_like(loss), torch.empty_like(dh), torch.empty_like(dgamma), torch.empty_like(W0))
            torch.cuda.synchronize()
            want = [e[0], e_hl, e[2], *e[3], n[0], n[1], n[2], n[3]]
            for a, b in zip(got, want):
                assert torch.equal(a.reshape(-1).view(torch.uint8), b.reshape(-1).view(torch.uint8))
    finally:
        flce.flce_set_logits_budget_bytes(old)


# ---- row compaction: rows with an ignored target are left out of the products ----

def _with_budget_rows(rows_per_chunk, V, fn):
    import paper_2410_10989_amd as flce
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(rows_per_chunk * ((V + 63) // 64 * 64) * 2)
        return fn()
    finally:
        flce.flce_set_logits_budget_bytes(old)


@pytest.mark.parametrize("frac", [0.9, 0.5, 0.26])
def test_mostly_ignored_rows_leave_leading_chunks_empty(frac):
    # 4 chunks of 256 rows are launched; the valid rows are dealt evenly to the last one(s), the
    # launches before them run with zero live rows (their dW launches return at once)
    import paper_2410_10989_amd as flce
    w = workloads.make(1024, 128, 1000, "bf16", ignore=("iid", frac), seed=900 + int(frac * 100),
                       name="sparse_targets")
    assert flce.flce_get_row_compaction()

    def run():
        assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16) == 4
        return check_full(w)
    _with_budget_rows(256, w.V, run)


def test_valid_rows_exactly_fill_the_chunks():
    import paper_2410_10989_amd as flce
    w = workloads.make(768, 64, 512, "bf16", seed=5, name="exact_fill")
    w.targets[np.arange(768) % 3 == 2] = w.ignore_index      # 512 valid rows = 2 chunks of 256
    assert w.n_valid == 512
    _with_budget_rows(256, w.V, lambda: check_full(w))


def test_all_rows_ignored_with_several_chunks():
    w = workloads.make(700, 64, 384, "bf16", seed=6, name="all_ignored_chunked")
    w.targets[:] = w.ignore_index

    def run():
        loss, dX, dW = run_gpu(w)
        assert loss == 0.0 and (to_host(dX) == 0).all() and (to_host(dW) == 0).all()
    _with_budget_rows(256, w.V, run)


def test_compaction_on_and_off_agree():
    # dX rows are computed by the same arithmetic either way (bitwise equal); dW sums the same
    # non-zero terms in other groups of K, the loss adds the same row losses in another order
    import paper_2410_10989_amd as flce
    w = workloads.make(1300, 256, 2048, "bf16", ignore=("pad", 100, 60), seed=77, name="on_off")
    on = run_gpu(w)
    try:
        flce.flce_set_row_compaction(False)
        off = run_gpu(w)
    finally:
        flce.flce_set_row_compaction(True)
    assert abs(on[0] - off[0]) <= 1e-6 * abs(off[0])
    assert torch.equal(on[1].view(torch.int16), off[1].view(torch.int16))
    err = (on[2].float() - off[2].float()).abs().max().item()
    assert err <= 2.0 ** -7 * off[2].float().abs().max().item()
    ref = oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    assert_close("dW (compaction off)", to_host(off[2]), ref.dW, TOL["bf16"][1])


def test_mfma_only_loop_runs_and_counts_its_flops():
    # measurement aid: zero operands give zero checksums, random operands finite ones
    import paper_2410_10989_amd as flce
    out = torch.full((8 * 256,), float("nan"), device="cuda")
    fl = flce.flce_mfma_ceiling_launch(0, 8, 10, 0.02, out)
    torch.cuda.synchronize()
    assert fl == 8 * 4 * 10 * 16 * 32768.0 and (out == 0).all()
    flce.flce_mfma_ceiling_launch(2, 8, 10, 0.02, out)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and (out != 0).any()
    with pytest.raises(flce.FlceError):
        flce.flce_mfma_ceiling_launch(2, 9, 10, 0.02, out)       # out too small


def test_options_passed_with_the_call_equal_the_setters():
    # three chunks without row compaction through flce_fwd_bwd_opt: the same bits as the same
    # settings made through the process-wide setters, which the call leaves untouched
    import paper_2410_10989_amd as flce
    w = workloads.make(700, 128, 1536, "bf16", ignore=("iid", 0.2), seed=31, name="options")
    X, W, t = upload(w)
    budget = 256 * 1536 * 2
    o = flce.flce_options(logits_budget_bytes=budget, row_compaction=False)
    loss_o, dX_o, dW_o = flce.flce_fwd_bwd_opt(X, W, t, o, w.ignore_index)
    torch.cuda.synchronize()
    assert flce.flce_get_logits_budget_bytes() == 0 and flce.flce_get_row_compaction()
    try:
        flce.flce_set_logits_budget_bytes(budget)
        flce.flce_set_row_compaction(False)
        assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16) == 3
        loss_s, dX_s, dW_s = run_gpu(w)
    finally:
        flce.flce_set_logits_budget_bytes(0)
        flce.flce_set_row_compaction(True)
    assert loss_o.item() == loss_s
    assert torch.equal(dX_o.view(torch.int16), dX_s.view(torch.int16))
    assert torch.equal(dW_o.view(torch.int16), dW_s.view(torch.int16))
    ref = oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    assert_close("dW", to_host(dW_o), ref.dW, TOL["bf16"][1])
    skip = flce.flce_options(flags=flce.SKIP_DX)
    loss_k, dX_k, dW_k = flce.flce_fwd_bwd_opt(X, W, t, skip, w.ignore_index)
    torch.cuda.synchronize()
    assert dX_k is None and abs(loss_k.item() - ref.loss) <= TOL["bf16"][0] * abs(ref.loss)


def test_calls_with_workspaces_of_their_own_may_overlap():
    # two different problems on two streams at the same time, each call with a workspace of its
    # own (flce_options): the same bits as the two calls one after the other on the shared
    # workspace.  The buffers start out full of NaN bit patterns: the call relies on nothing in them.
    import paper_2410_10989_amd as flce
    ws_a = workloads.make(1500, 256, 3000, "bf16", ignore=("iid", 0.2), seed=41, name="own_ws_a")
    ws_b = workloads.make(900, 256, 5000, "bf16", targets="zipf", ignore=("pad", 128, 40), seed=42, name="own_ws_b")
    budget = 512 * 3000 * 2                                    # several chunks each
    seq, ins = [], []
    try:
        flce.flce_set_logits_budget_bytes(budget)
        for w in (ws_a, ws_b):
            X, W, t = upload(w)
            ins.append((X, W, t))
            seq.append(flce.flce_fwd_bwd(X, W, t, w.ignore_index))
        torch.cuda.synchronize()
    finally:
        flce.flce_set_logits_budget_bytes(0)
    streams = [torch.cuda.Stream() for _ in range(2)]
    opts, outs = [], []
    for w in (ws_a, ws_b):
        need = flce.flce_workspace_bytes_opt(w.BT, w.H, w.V, flce.FLCE_BF16, flce.flce_options(logits_budget_bytes=budget))
        buf = torch.full((need // 2 + 128,), -1, dtype=torch.int16, device="cuda")
        off = (-buf.data_ptr() % 256) // 2
        opts.append(flce.flce_options(logits_budget_bytes=budget, workspace=buf[off:off + need // 2]))
    torch.cuda.synchronize()
    for rep in range(3):                                       # the launches of the two calls interleave
        outs = []
        for (X, W, t), w, o, st in zip(ins, (ws_a, ws_b), opts, streams):
            outs.append(flce.flce_fwd_bwd_opt(X, W, t, o, w.ignore_index, stream=st))
        torch.cuda.synchronize()
        for (l1, dx1, dw1), (l2, dx2, dw2) in zip(seq, outs):
            assert l1.item() == l2.item()
            assert torch.equal(dx1.view(torch.int16), dx2.view(torch.int16))
            assert torch.equal(dw1.view(torch.int16), dw2.view(torch.int16))
    ref = oracle.flce(ws_b.X, ws_b.W, ws_b.targets, ws_b.ignore_index)
    assert_close("dW", to_host(outs[1][2]), ref.dW, TOL["bf16"][1])
    assert_close("dX", to_host(outs[1][1]), ref.dX, TOL["bf16"][1])
    # a buffer one byte short is refused before anything is launched
    w, (X, W, t) = ws_a, ins[0]
    need = flce.flce_workspace_bytes_opt(w.BT, w.H, w.V, flce.FLCE_BF16, flce.flce_options(logits_budget_bytes=budget))
    short = flce.flce_options(logits_budget_bytes=budget, workspace=opts[0]._workspace_tensor[:need // 2 - 1])
    with pytest.raises(flce.FlceError) as e:
        flce.flce_fwd_bwd_opt(X, W, t, short, w.ignore_index)
    assert e.value.status == 5


@pytest.mark.parametrize("chunks", [1, 2, 3])
def test_dw_last_round_of_tiles_is_cut_along_k(chunks):
    # dW has 65 x 4 = 260 output tiles: 33 per XCD, i.e. one more than a round of 32 CUs, so the
    # last tile of every XCD's span is cut into K ranges (fp32 partial blocks, fixed-order sum by
    # a second launch).  One chunk: the sum is written as bf16; two chunks: fp32 partial sums of
    # dW across the chunks, the tail tiles of both launches go through the same reduction; three:
    # the middle launch adds fp32 to fp32
    import paper_2410_10989_amd as flce
    w = workloads.make(2048 * max(chunks, 2), 1024, 16640, "bf16", targets="zipf", ignore=("iid", 0.1),
                       seed=260 + chunks, name="dw_tail")
    old = flce.flce_get_logits_budget_bytes()
    try:
        if chunks >= 2:
            flce.flce_set_logits_budget_bytes(2048 * 16640 * 2)
        # (the rows that have a target are dealt evenly to the chunks, 10 % fewer than 2048 each)
        assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16) == chunks
        check_full(w)
    finally:
        flce.flce_set_logits_budget_bytes(old)


@pytest.mark.parametrize("compaction", [True, False])
def test_dw_cut_last_round_with_empty_and_ragged_chunks(compaction):
    # the same dW shape in 3 chunks of 2048 rows at most.  Row compaction on: 70 % of the targets
    # are ignored, so the first launch has no live rows and returns at once, together with its
    # second, summing launch; the live launches see fewer K steps than the plan assumed.  Off: the
    # last chunk has 1904 rows, too few K steps for two ranges: that launch is not cut, the others are
    import paper_2410_10989_amd as flce
    w = workloads.make(6000, 1024, 16640, "bf16", targets="zipf", ignore=("iid", 0.7 if compaction else 0.1),
                       seed=271 + int(compaction), name="dw_tail_ragged")
    old, old_c = flce.flce_get_logits_budget_bytes(), flce.flce_get_row_compaction()
    try:
        flce.flce_set_logits_budget_bytes(2048 * 16640 * 2)
        flce.flce_set_row_compaction(compaction)
        assert flce.flce_num_chunks(w.BT, w.H, w.V, flce.FLCE_BF16) == 3
        check_full(w)
    finally:
        flce.flce_set_logits_budget_bytes(old)
        flce.flce_set_row_compaction(old_c)
