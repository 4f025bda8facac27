"""Parity of the RMSNorm + fused linear cross-entropy entry point with the fp64
CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads
from flce_testlib import TOL, assert_close, assert_loss, to_device, to_host
from oracle import flce_oracle as oracle

pytestmark = pytest.mark.gpu


def make_case(BT, H, V, dtype, seed, ignore=("iid", 0.1)):
    # raw hidden states with a spread of row scales; gamma close to one
    w = workloads.make(BT, H, V, dtype, ignore=ignore, seed=seed, name="rmsnorm", x_std=2.5)
    g = np.random.Generator(np.random.Philox(key=[seed, 99]))
    gamma = (1.0 + 0.2 * g.standard_normal(H)).astype(np.float32)
    scale = np.exp(g.standard_normal(BT)).astype(np.float32)[:, None]
    h = (w.X * scale).astype(np.float32)
    if dtype == "bf16":
        workloads.round_to_bf16(gamma)
        workloads.round_to_bf16(h)
    return w, h, gamma


def check(w, h, gamma, eps=1e-6, flags=0):
    import paper_2410_10989_amd as flce
    print(f"case rmsnorm BT={w.BT} H={w.H} V={w.V} {w.dtype} seed={w.seed} flags={flags}", flush=True)
    ref = oracle.rmsnorm_flce(h, gamma, eps, w.W, w.targets, w.ignore_index)
    hd, gd, Wd = to_device(h, w.dtype), to_device(gamma, w.dtype), to_device(w.W, w.dtype)
    t = torch.from_numpy(w.targets).cuda()
    nan = float("nan")
    dh, dg, dW = torch.full_like(hd, nan), torch.full_like(gd, nan), torch.full_like(Wd, nan)
    loss = torch.full((), nan, dtype=torch.float32, device="cuda")
    flce.flce_rmsnorm_fwd_bwd(hd, gd, eps, Wd, t, w.ignore_index, loss=loss, dh=dh, dgamma=dg, dW=dW,
                              flags=flags)
    torch.cuda.synchronize()
    rl, rg = TOL[w.dtype]
    assert_loss(float(loss.item()), ref.loss, rl)
    if not flags & flce.SKIP_DX:
        assert_close("dh", to_host(dh), ref.dh, rg)
        assert_close("dgamma", to_host(dg), ref.dgamma, rg)
        ign = w.targets == w.ignore_index
        assert (to_host(dh)[ign] == 0).all()
    else:
        assert torch.isnan(dh.float()).all() and torch.isnan(dg.float()).all()
    if not flags & flce.SKIP_DW:
        assert_close("dW", to_host(dW), ref.dW, rg)
    else:
        assert torch.isnan(dW.float()).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("BT,H,V", [
    (768, 320, 1344),    # tuned kernels
    (300, 136, 1000),    # guarded kernels, ragged
    (77, 100, 333),      # H not a multiple of anything useful
    (600, 1024, 512),    # more rows than backward workgroups: several rows per partial-sum slot
    (520, 2560, 256),    # two (bf16) or four (fp32) 16-byte vectors per thread in the row kernels
    (300, 4104, 128),    # four vectors per thread, last one partly used (bf16); scalar form (fp32)
])
def test_rmsnorm_head_matches_oracle(dtype, BT, H, V):
    check(*make_case(BT, H, V, dtype, seed=500 + BT + H))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rmsnorm_head_with_several_chunks(dtype):
    import paper_2410_10989_amd as flce
    old = flce.flce_get_logits_budget_bytes()
    try:
        flce.flce_set_logits_budget_bytes(256 * 1536 * (2 if dtype == "bf16" else 4))
        code = flce.FLCE_BF16 if dtype == "bf16" else flce.FLCE_F32
        assert flce.flce_num_chunks(513, 192, 1536, code) == 3
        # the normalised rows exist one chunk at a time: extra workspace does not grow with BT
        assert flce.flce_rmsnorm_workspace_bytes(256 * 80, 192, 1536, code) == \
            flce.flce_rmsnorm_workspace_bytes(256 * 40, 192, 1536, code)
        check(*make_case(513, 192, 1536, dtype, seed=4243, ignore=("iid", 0.15)))
    finally:
        flce.flce_set_logits_budget_bytes(old)


@pytest.mark.parametrize("flag", ["SKIP_DX", "SKIP_DW"])
def test_rmsnorm_head_frozen_sides(flag):
    import paper_2410_10989_amd as flce
    check(*make_case(512, 256, 2048, "bf16", seed=77), flags=getattr(flce, flag))


def test_large_eps_is_applied_inside_the_root():
    check(*make_case(256, 128, 640, "f32", seed=3), eps=0.75)
