"""Host-side checks that need no GPU: the C-ABI library loads, exports every
symbol the header declares, rejects bad arguments before touching the device,
and the chunk scheduler keeps the workspace bounded independently of BT."""
import ctypes
import os
import re

import pytest

import paper_2410_10989_amd as flce

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flce.h")).read()
    return sorted(set(re.findall(r"FLCE_API[^;(]*?\b(flce_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 14 and "flce_fwd_bwd" in names
    L = flce.lib()
    for n in names:
        assert hasattr(L, n), f"libflce.so does not export {n}"


def test_paper_chunk_rule_at_the_five_shapes():
    # 2^ceil(log2(ceil(BT / ceil(V/H)))): paper section 3.2, FLCE paragraph.
    shapes = [(256, 512, 4096), (4096, 4096, 32000), (8192, 4096, 128256),
              (16384, 3584, 152064), (8192, 2304, 256000)]
    assert [flce.flce_paper_chunk_rows(*s) for s in shapes] == [32, 512, 256, 512, 128]
    assert flce.flce_paper_chunk_rows(1, 8, 8) == 1
    assert flce.flce_paper_chunk_rows(100, 10, 10) == 128


def test_memory_example_printed_in_the_paper():
    vals = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_values.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    n = flce.flce_full_logits_bytes(int(vals["logits_example_batch"] * vals["logits_example_seq"]),
                                    int(vals["logits_example_vocab"]), flce.FLCE_BF16)
    assert n == 8 * 4096 * 256000 * 2
    assert round(n / 1e9, 1) == vals["logits_example_gigabytes"]


@pytest.mark.parametrize("H,V", [(4096, 128256), (3584, 152064), (2304, 256000), (4096, 32000)])
def test_workspace_is_bounded_independently_of_BT(H, V):
    code = flce.FLCE_BF16
    cap = flce.flce_workspace_bytes_max(H, V, code)
    C = flce.flce_chunk_rows(10 ** 7, H, V, code)
    sizes = [flce.flce_workspace_bytes(bt, H, V, code) for bt in (C, 2 * C, 4 * C, 8 * C, 64 * C)]
    assert all(0 < s <= cap for s in sizes)
    # A batch whose whole logits take no more memory than one chunk plus the fp32 dW partial
    # sums of a chunked run is not chunked at all (smaller and faster); beyond that the
    # workspace is constant
    single_rows = (max(1 << 30, 4096 * V * 2) + V * H * 4) // (V * 2)
    for bt in (single_rows - 300, single_rows):
        assert flce.flce_num_chunks(bt, H, V, code) == 1
        assert flce.flce_workspace_bytes(bt, H, V, code) <= cap
    assert flce.flce_num_chunks(single_rows + 1, H, V, code) > 1
    many = [flce.flce_workspace_bytes(bt, H, V, code) for bt in (single_rows + 1, 4 * C, 8 * C, 64 * C, 4096 * C)
            if bt % C == 0 or bt == single_rows + 1]
    assert len(set(many[1:])) == 1 and all(s <= cap for s in many)
    # a chunk whose row count is not a multiple of 64 takes the guarded kernels, which
    # need transposed scratch: larger, but still bounded by the same cap for any BT
    ragged = [flce.flce_workspace_bytes(bt, H, V, code) for bt in (C + 1, 9 * C + 3, 10 ** 7 + 1)]
    assert all(0 < s <= cap for s in ragged)
    assert flce.flce_get_logits_budget_bytes() == 0      # automatic: 1 GiB or 4096 rows
    budget = max(1 << 30, 4096 * V * 2)
    assert C % 256 == 0 and C * V * 2 <= budget and C >= 4096
    for bt in (1, 255, C, C + 1, 3 * C - 5):
        c, n = flce.flce_chunk_rows(bt, H, V, code), flce.flce_num_chunks(bt, H, V, code)
        assert c * n >= bt > c * (n - 1) and (c <= max(C, 256) or (n == 1 and c <= single_rows))
        assert flce.flce_workspace_bytes(bt, H, V, code) <= cap


def test_dx_product_is_cut_along_k_to_fill_whole_rounds_of_cus():
    code = flce.FLCE_BF16
    k = flce.flce_dx_k_ranges
    assert k(8192, 4096, 128256, code) == 1       # 2 chunks of 4096 rows: 16 x 16 = 256 tiles, one full round
    assert k(4352, 4096, 8192, code) == 2         # 272 tiles, K = 128 steps: at most 2 ranges of 64 steps
    assert k(16384, 3584, 152064, code) >= 4      # chunks of 3328 rows: 13 x 14 = 182 tiles
    assert k(8192, 2304, 256000, code) >= 3       # chunks of 2048 rows: 8 x 9 = 72 tiles
    assert k(65536, 4096, 32000, code) == 1       # 16384-row chunks: 1024 tiles, many rounds
    assert k(256, 512, 4096, flce.FLCE_F32) == 16 # guarded kernels (fp32 storage): 2 x 4 tiles of 128 x 128
    assert k(4096, 4096, 32000, flce.FLCE_F32) == 1
    for bt, h, v in [(4352, 4096, 8192), (16384, 3584, 152064), (8192, 2304, 256000)]:
        # the fp32 partial results are part of the reported workspace and stay within the budget
        c = flce.flce_chunk_rows(bt, h, v, code)
        part = k(bt, h, v, code) * c * h * 4
        assert part <= max(1 << 30, 4096 * ((v + 63) // 64 * 64) * 2)
        assert flce.flce_workspace_bytes(bt, h, v, code) >= part


def test_bad_arguments_are_rejected_on_the_host():
    L = flce.lib()
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    ok = dict(X=a, W=a + 256, t=a + 512, loss=a + 768, dX=a + 1024, dW=a + 1280)

    def call(BT=4, H=8, V=16, ign=-100, dtype=1, **kw):
        p = dict(ok, **kw)
        return L.flce_fwd_bwd(p["X"], p["W"], p["t"], BT, H, V, ign, dtype, p["loss"], p["dX"],
                              p["dW"], None)

    assert call(X=None) == 1 and call(dW=None) == 1 and call(loss=None) == 1
    assert call(BT=0) == 2 and call(V=-1) == 2 and call(H=2 ** 40) == 2
    assert call(dtype=7) == 3
    assert call(X=a + 2) == 4 and call(t=a + 516) == 4
    assert call(ign=3) == 7
    assert L.flce_fwd_bwd_ex(ok["X"], ok["W"], ok["t"], 4, 8, 16, -100, 1, ok["loss"], None, None,
                             64, None) == 7
    # several heads: host arrays of device pointers
    P2 = ctypes.c_void_p * 2
    Ws, ts, dWs = P2(a + 256, a + 1536), P2(a + 512, a + 512), P2(a + 1280, a + 1792)

    def heads(n=2, W=Ws, t=ts, dW=dWs, wts=None, flags=0):
        return L.flce_multihead_fwd_bwd(a, W, t, wts, n, 4, 8, 16, -100, 1, a + 768, None, a + 1024,
                                        dW, flags, None)

    F2 = ctypes.c_float * 2
    assert heads(n=0) == 7 and heads(n=17) == 7
    assert heads(W=P2(a + 256, None)) == 1 and heads(dW=None) == 1 and heads(t=None) == 1
    assert heads(dW=P2(a + 1280, a + 1280)) == 7              # heads sharing one dW
    assert heads(wts=F2(1.0, float("nan"))) == 7 and heads(wts=F2(float("inf"), 1.0)) == 7
    assert heads(W=P2(a + 256, a + 1538)) == 4
    assert heads(flags=8) == 7
    # RMSNorm in front of the projection
    cf = ctypes.c_float

    def norm(h=a, gamma=a + 2048, eps=1e-6, dh=a + 1024, dg=a + 2304, dW=a + 1280, flags=0):
        return L.flce_rmsnorm_fwd_bwd(h, gamma, cf(eps), a + 256, a + 512, 4, 8, 16, -100, 1, a + 768,
                                      dh, dg, dW, flags, None)

    assert norm(gamma=None) == 1 and norm(dg=None) == 1 and norm(dh=None) == 1
    assert norm(gamma=a + 2049) == 4 and norm(h=a + 4) == 4
    assert norm(eps=-1.0) == 7 and norm(eps=float("nan")) == 7 and norm(eps=float("inf")) == 7
    assert norm(flags=4) == 7
    assert L.flce_cross_entropy_inplace(None, a, 1, 1, 1, -100, 1, a, None) == 1
    assert L.flce_cross_entropy_inplace(a, a, 4, 16, 8, -100, 1, a, None) == 2   # ldz < V
    # the MFMA-only measurement loop
    assert L.flce_mfma_ceiling_launch(2, 256, 100, cf(0.02), None, 65536, None) == 1
    for bad in [(3, 256, 100, 65536), (2, 0, 100, 65536), (2, 256, 0, 65536), (2, 256, 100, 65535),
                (2, 70000, 100, 1 << 30), (2, 256, (1 << 18) + 1, 65536)]:
        assert L.flce_mfma_ceiling_launch(bad[0], bad[1], bad[2], cf(0.02), a, bad[3], None) == 7
    assert L.flce_mfma_ceiling_launch(2, 256, 100, cf(float("nan")), a, 65536, None) == 7
    for s in range(8):
        assert flce.status_string(s) not in ("", "unknown status")


def test_binding_refuses_cpu_tensors():
    import torch
    X = torch.zeros(4, 8, dtype=torch.bfloat16)
    W = torch.zeros(16, 8, dtype=torch.bfloat16)
    t = torch.zeros(4, dtype=torch.int64)
    with pytest.raises(ValueError):
        flce.flce_fwd_bwd(X, W, t, loss=torch.zeros(()), dX=X.clone(), dW=W.clone())


def test_options_passed_with_the_call_plan_like_the_setters():
    code = flce.FLCE_BF16
    H, V = 4096, 128256
    o = flce.flce_options()
    assert o.size == ctypes.sizeof(flce.FlceOptions) and o.logits_budget_bytes == 0 and o.row_compaction == 1
    assert flce.flce_workspace_bytes_opt(8192, H, V, code, o) == flce.flce_workspace_bytes(8192, H, V, code)
    lit = flce.flce_options(logits_budget_bytes=1 << 30)          # a budget taken literally: two chunks
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(1 << 30)
        want = flce.flce_workspace_bytes(8192, H, V, code)
    finally:
        flce.flce_set_logits_budget_bytes(old)
    assert flce.flce_workspace_bytes_opt(8192, H, V, code, lit) == want != flce.flce_workspace_bytes(8192, H, V, code)
    assert flce.flce_get_logits_budget_bytes() == old              # the call's options leave the process-wide ones alone
    bad = flce.flce_options()
    bad.size = 8
    assert flce.flce_workspace_bytes_opt(8192, H, V, code, bad) == 0
    L = flce.lib()
    buf = (ctypes.c_char * 4096)()
    a = ctypes.addressof(buf)
    a += (-a) % 256
    assert L.flce_fwd_bwd_opt(a, a + 256, a + 512, 4, 8, 16, -100, 1, a + 768, a + 1024, a + 1280,
                              ctypes.byref(bad), None) == 7
    bad = flce.flce_options()
    bad.row_compaction = 5
    assert L.flce_fwd_bwd_opt(a, a + 256, a + 512, 4, 8, 16, -100, 1, a + 768, a + 1024, a + 1280,
                              ctypes.byref(bad), None) == 7
    # a workspace of the call's own: refused on the host when misaligned or too small
    need = flce.flce_workspace_bytes_opt(4, 8, 16, code, flce.flce_options())
    assert need > 0
    own = flce.flce_options()
    assert not own.workspace and own.workspace_bytes == 0
    own.workspace, own.workspace_bytes = a + 2048 + 8, 1 << 30
    assert L.flce_fwd_bwd_opt(a, a + 256, a + 512, 4, 8, 16, -100, 1, a + 768, a + 1024, a + 1280,
                              ctypes.byref(own), None) == 4
    own.workspace, own.workspace_bytes = a + 2048, need - 1
    assert L.flce_fwd_bwd_opt(a, a + 256, a + 512, 4, 8, 16, -100, 1, a + 768, a + 1024, a + 1280,
                              ctypes.byref(own), None) == 5


def test_budget_for_a_workspace_of_a_given_size():
    code = flce.FLCE_BF16
    BT, H, V = 131072, 4096, 128256
    ldz = (V + 63) // 64 * 64
    old = flce.flce_get_logits_budget_bytes()
    try:
        last_rows = None
        for cap in (1 << 30, 3 << 30, 4 << 30, 8 << 30, 64 << 30):
            b = flce.flce_logits_budget_for_workspace(BT, H, V, code, cap)
            if cap == 1 << 30:
                assert b == 0          # the fp32 dW partial sums alone are 2.1 GB
                continue
            assert b > 0 and b % (256 * ldz * 2) == 0
            flce.flce_set_logits_budget_bytes(b)
            rows = flce.flce_chunk_rows(BT, H, V, code)
            assert rows * ldz * 2 <= b or rows == BT      # (chunks are evened out below the budget's row count)
            assert flce.flce_workspace_bytes(BT, H, V, code) <= cap
            flce.flce_set_logits_budget_bytes(b + 256 * ldz * 2)      # one step more does not fit
            assert rows >= BT or flce.flce_workspace_bytes(BT, H, V, code) > cap
            assert last_rows is None or rows >= last_rows
            last_rows = rows
        assert last_rows == BT             # 64 GiB: the whole batch as one chunk
    finally:
        flce.flce_set_logits_budget_bytes(old)
    assert flce.flce_logits_budget_for_workspace(0, H, V, code, 1 << 40) == 0
