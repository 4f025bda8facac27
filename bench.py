"""Benchmark of the fused linear cross-entropy forward+backward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]

One step = one pass of the whole hot path (count, chunked logits GEMM, in-place
cross entropy, dX GEMM, dW GEMM, finalize) over one synthetic batch that is
already resident in HBM.  Prints ONE JSON line: tokens/s for forward+backward,
the roofline of the dominant kernel (per-launch algorithmic flops over its
average launch time, HIP events on the launch stream), and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense matrix peaks
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel (logits product at config 3) from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, each scaled by what
# the same counter reads for the 1 GiB copy of --calibrate-copy; the summary of
# those runs is profiles/gemm_bf16_256_config3_hbm_traffic.txt.  Only valid for
# the default workload.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 9.35e9


def bench_cross_entropy(args):
    """Stand-alone cross entropy forward+backward (logits given, gradient written in
    place) at the vocabulary sizes of the paper's kernel benchmark (section 4.1:
    40960 ... 163840), bf16 logits, 4096 rows.  HBM-bound: the algorithmic traffic
    is one read and one write of the logits."""
    import torch

    import paper_2410_10989_amd as flce

    BT = 4096
    rows = []
    for V in (40960, 81920, 122880, 163840):
        g = torch.Generator(device="cuda").manual_seed(241010989 + V)
        Z0 = (torch.randn(BT, V, generator=g, device="cuda") * 1.3).to(torch.bfloat16)
        t = torch.randint(0, V, (BT,), generator=g, device="cuda")
        t[::10] = -100
        Z = torch.empty_like(Z0)
        loss = torch.empty((), dtype=torch.float32, device="cuda")
        times = []
        for it in range(args.warmup + args.steps):
            Z.copy_(Z0)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flce.flce_cross_entropy_inplace(Z, t, -100, loss=loss)
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                times.append(e0.elapsed_time(e1))
        times.sort()
        med = times[len(times) // 2]
        algo_bytes = 2.0 * BT * V * 2
        rows.append({"V": V, "ms_median": med, "ms_q20": times[int(0.2 * (len(times) - 1))],
                     "ms_q80": times[int(0.8 * (len(times) - 1))],
                     "algorithmic_gbs": algo_bytes / (med * 1e-3) / 1e9,
                     "frac_of_hbm_peak": algo_bytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "loss": float(loss.item())})
        del Z0, Z
    head = rows[-1]
    print(json.dumps({
        "metric": "cross entropy fwd+bwd tokens/s (logits given, in-place gradient)",
        "value": BT / (head["ms_median"] * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_median"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "standalone_ce:BT=4096,V=163840 (headline of the sweep)", "BT": BT},
        "roofline": {"bound": "hbm", "achieved": head["algorithmic_gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": head["frac_of_hbm_peak"], "traffic": None},
        "sweep": rows}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="workload 1-5 (3 = Llama-3-8B lm_head)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-rows", type=int, default=1024)
    ap.add_argument("--budget-mib", type=int, default=0, help="logits chunk budget override")
    ap.add_argument("--mode", choices=("flce", "ce"), default="flce",
                    help="flce: the fused path (default); ce: stand-alone cross entropy on given "
                         "logits, swept over the vocabulary sizes of the paper's kernel benchmark")
    ap.add_argument("--heads", type=int, default=1,
                    help="> 1: that many decoding heads on the shared hidden states (the paper's "
                         "Medusa setting, section 4.2), timed through flce_multihead_fwd_bwd")
    ap.add_argument("--skip-dx", action="store_true",
                    help="frozen backbone (Medusa stage 1): no hidden-state gradient")
    ap.add_argument("--no-compaction", action="store_true",
                    help="project every row, also those with an ignored target (A/B of the row compaction)")
    ap.add_argument("--rmsnorm", action="store_true",
                    help="time flce_rmsnorm_fwd_bwd: RMSNorm of raw hidden states fused in front (one head)")
    ap.add_argument("--no-mfma-loop", action="store_true",
                    help="skip the MFMA-only loop that is reported beside the roofline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one plain 1 GiB device copy first (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path is a single-GPU kernel "
              "pipeline; no collectives are part of it). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2410_10989_amd as flce
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.mode == "ce":
        return bench_cross_entropy(args)
    if args.budget_mib:
        flce.flce_set_logits_budget_bytes(args.budget_mib << 20)
    if args.no_compaction:
        flce.flce_set_row_compaction(False)

    t0 = time.time()
    w = workloads.make_config(args.config)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    code = flce.FLCE_BF16 if w.dtype == "bf16" else flce.FLCE_F32

    def up(a):
        if w.dtype == "bf16":
            return torch.from_numpy(workloads.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    X, W, t = up(w.X), up(w.W), torch.from_numpy(w.targets).cuda()
    dX, dW = torch.empty_like(X), torch.empty_like(W)
    loss = torch.empty((), dtype=torch.float32, device="cuda")
    print(f"# inputs {w.name} BT={w.BT} H={w.H} V={w.V} {w.dtype} generated+uploaded in "
          f"{time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # 1 GiB read + 1 GiB written by one copy kernel
        torch.cuda.synchronize()
        del src, dst

    nh = args.heads
    flags = flce.SKIP_DX if args.skip_dx else 0
    if nh > 1:
        # extra heads: seeded N(0, 0.02^2) weights drawn on the device; head j's target at
        # position p is head 0's target at p + j inside sequences of 2048 tokens
        seq = 2048
        Ws, ts, dWs = [W], [t], [dW]
        pos = torch.arange(w.BT, device="cuda") % seq
        for j in range(1, nh):
            g = torch.Generator(device="cuda").manual_seed(w.seed + 16 + j)
            Ws.append((torch.randn(w.V, w.H, generator=g, device="cuda") * 0.02).to(tdt))
            tj = torch.roll(t, -j)
            tj[pos >= seq - j] = w.ignore_index
            ts.append(tj)
            dWs.append(torch.empty_like(W))
        wts = [0.8 ** j for j in range(nh)]
        hl = torch.empty(nh, dtype=torch.float32, device="cuda")

        def step():
            flce.flce_multihead_fwd_bwd(X, Ws, ts, wts, w.ignore_index, loss=loss, head_losses=hl,
                                        dX=None if args.skip_dx else dX, dWs=dWs, flags=flags)
    elif args.rmsnorm:
        h_np, gamma_np = workloads.make_rmsnorm_inputs(w)
        hraw, gamma = up(h_np), up(gamma_np)
        dgamma = torch.empty_like(gamma)

        def step():
            flce.flce_rmsnorm_fwd_bwd(hraw, gamma, 1e-6, W, t, w.ignore_index, loss=loss,
                                      dh=None if args.skip_dx else dX,
                                      dgamma=None if args.skip_dx else dgamma, dW=dW, flags=flags)
    else:
        def step():
            flce.flce_fwd_bwd(X, W, t, w.ignore_index, loss=loss, dX=None if args.skip_dx else dX,
                              dW=dW, flags=flags)

    # rows that are actually projected: with row compaction (the default) only the rows that
    # have a target, summed over the heads
    all_targets = ts if nh > 1 else [t]
    compaction = flce.flce_get_row_compaction() and w.dtype == "bf16" and w.H % 64 == 0
    rows_projected = sum(int((x != w.ignore_index).sum().item()) for x in all_targets) if compaction \
        else w.BT * nh

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    flce.flce_timing_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    marks[0].record()
    for k in range(args.steps):
        step()
        marks[k + 1].record()      # same stream as the call: per-step times for the quantiles
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    quantile = lambda q: per_step[int(round(q * (len(per_step) - 1)))]
    flce.flce_timing_enable(False)
    kt = flce.flce_timing_collect()
    ms_per_step = (t2 - t1) * 1e3 / args.steps
    tokens_per_s = w.BT / (ms_per_step * 1e-3)

    flops_step = (4.0 if args.skip_dx else 6.0) * w.BT * w.H * w.V * nh
    tflops = flops_step / (ms_per_step * 1e-3) / 1e12
    peak = MFMA_PEAK_TFLOPS[w.dtype]

    # Dominant kernel = the kernel symbol with the largest total time.  The logits and
    # dX products are one symbol each; with several chunks the dW product runs as
    # two symbols (fp32 partial sums, then the bf16 result), so its time is split.
    nchunks = flce.flce_num_chunks(w.BT, w.H, w.V, code)
    gemm_kinds = ("logits_gemm", "dw_gemm") if args.skip_dx else ("logits_gemm", "dx_gemm", "dw_gemm")
    symbols = {"logits_gemm": 1, "dx_gemm": 1, "dw_gemm": 2 if nchunks > 1 else 1}
    dom = max(gemm_kinds, key=lambda k: kt[k][0] / symbols[k])
    dom_ms, dom_n = kt[dom]
    # executed flops of the dominant kernel, mean over its launches (ignored rows are not projected)
    flops_per_launch = 2.0 * rows_projected * w.H * w.V * args.steps / max(dom_n, 1)
    dom_avg_ms = dom_ms / max(dom_n, 1)
    achieved = flops_per_launch / (dom_avg_ms * 1e-3) / 1e12 if dom_n else 0.0
    ce_ms, ce_n = kt["ce_rows"]
    ce_gbs = (2.0 * w.BT * w.V * (2 if w.dtype == "bf16" else 4) * args.steps) / (ce_ms * 1e-3) / 1e9 if ce_n else 0.0

    out = {
        "metric": ("RMSNorm + " if args.rmsnorm else "") +
                  ("FLCE fwd+bwd tokens/s" if nh == 1 and not args.skip_dx else
                   f"FLCE fwd+bwd tokens/s, {nh} head(s)" + (", no dX" if args.skip_dx else "")),
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_q20_median_q80": [quantile(0.2), quantile(0.5), quantile(0.8)],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"config{args.config}:{w.name}", "BT": w.BT, "H": w.H, "V": w.V,
                   "ignore_frac": round(1 - w.n_valid / w.BT, 4), "chunk_rows":
                   flce.flce_chunk_rows(w.BT, w.H, w.V, code), "chunks": nchunks,
                   "logits_budget_mib": (flce.flce_get_logits_budget_bytes() >> 20) or "auto"},
        "heads": nh,
        "tflops_over_6BTHV": tflops,   # nominal: over 6*BT*H*V per head (4*BT*H*V without dX)
        "mfma_util_frac_of_peak": tflops / peak,
        # rows with an ignored target are left out of the products (row compaction): what the
        # matrix cores really executed is smaller than the nominal count by this share
        "row_compaction": bool(compaction),
        "rows_projected": rows_projected,
        "tflops_executed": tflops * rows_projected / (w.BT * nh),
        "peak_extra_hbm_mb": (flce.flce_rmsnorm_workspace_bytes if args.rmsnorm else
                              flce.flce_workspace_bytes)(w.BT, w.H, w.V, code) / 1e6,
        "full_logits_avoided_mb": flce.flce_full_logits_bytes(w.BT, w.V, code) / 1e6,
        "loss": float(loss.item()),
        "kernel_ms_per_step": {k: kt[k][0] / args.steps for k in kt},
        "ce_rows_hbm_gbs": ce_gbs,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": peak,
                     "unit": "TFLOP/s", "frac": achieved / peak,
                     "avg_launch_ms": dom_avg_ms, "launches": dom_n,
                     "flops_per_launch": flops_per_launch,
                     # the same with the nominal count (every row of the batch, ignored or not)
                     "achieved_nominal": achieved * (w.BT * nh) / rows_projected,
                     "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH
                     if args.config == 3 and dom == "logits_gemm" and not args.budget_mib else None},
    }

    if w.dtype == "bf16" and not args.no_mfma_loop:
        # What the matrix pipes sustain with nothing to feed them from memory: the same MFMA
        # instruction in a loop on register operands, one wavefront per SIMD, launches about
        # as long as a product launch.  On operands like the workload's (normal deviates,
        # 4 x 4 fragments per K sub-step) the chip clocks far lower than on zeros.
        scratch = torch.empty(256 * 256, dtype=torch.float32, device="cuda")

        def mfma_loop(pattern):
            # a train of launches back to back, as long as a few passes of the path: the clock
            # settles within the first launches, which are left out
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fl = 0.0
            for k in range(16):
                if k == 4:
                    e0.record()
                one = flce.flce_mfma_ceiling_launch(pattern, 256, 8000, 0.02, scratch)
                fl += one if k >= 4 else 0.0
            e1.record()
            e1.synchronize()
            return fl / (e0.elapsed_time(e1) * 1e-3) / 1e12

        rnd, zero = mfma_loop(2), mfma_loop(0)
        out["mfma_only_loop"] = {
            "random_operands_tflops": rnd, "zero_operands_tflops": zero,
            "what": "v_mfma_f32_32x32x16_bf16 on register operands, no memory traffic, 256 workgroups x 4 "
                    "wavefronts, 12 launches of ~3 ms back to back after 4 to settle the clock; random = N(0,1) x N(0,0.02^2) fragments, 4 A x 4 B per 16 MFMAs"}
        out["roofline"]["frac_of_mfma_only_loop_random"] = achieved / rnd if rnd > 0 else None

    if not args.no_cpu_baseline:
        from oracle import flce_oracle
        n = min(args.cpu_sample_rows, w.BT)
        tc = time.perf_counter()
        flce_oracle.flce(w.X[:n], w.W, w.targets[:n], w.ignore_index)
        dt = (time.perf_counter() - tc) * nh    # every head costs the oracle the same again
        out["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": flce_oracle.threads(),
                               "kind": "oracle",
                               "sample": f"first {n} of {w.BT} rows of the same workload, full fp64 "
                                         f"forward+backward, {dt:.1f} s"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
