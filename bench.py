"""Benchmark of the fused linear cross-entropy forward+backward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]

One step = one pass of the whole hot path (count, chunked logits GEMM, in-place
cross entropy, dX GEMM, dW GEMM, finalize) over one synthetic batch that is
already resident in HBM.  Prints ONE JSON line:

  value / ms_per_step    K passes in the library's default configuration, timed
                         with per-kernel timing OFF (wall clock around a synchronised
                         loop); socket power sampled meanwhile
  product_rooflines      a second, short loop with the library's per-kernel HIP events
                         on: per product class (logits, dX, dW) the executed flops per
                         launch over the mean launch time; `roofline` is the class that
                         takes the most time per step
  dense                  the same workload with row compaction off (every row projected,
                         as the paper does)
  per_config             all five benchmark workloads, about 0.3 s of passes each
  memory                 workspace against the full logits for growing BT
  mfma_only_loop         the MFMA instruction alone on register operands, with power
  cpu_baseline           the CPU oracle on a bounded sample of the same workload
"""
import argparse
import glob
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense matrix peaks
HBM_PEAK_GBS = 8000.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_bf16_256_config3_hbm_traffic.txt")


def measured_traffic_bytes():
    """HBM-side bytes per launch of each product class at the default workload, from the
    committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE runs, each scaled by
    what the same counter reads for a plain copy of known size): the line
    '# bench.py: traffic_bytes_per_launch logits=... dx=... dw=...' of that file."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return {}
    m = re.search(r"traffic_bytes_per_launch\s+(.*)", text)
    if not m:
        return {}
    return {k: float(v) for k, v in re.findall(r"(\w+)=([0-9.eE+]+)", m.group(1))}


class PowerSampler:
    """Socket power of the GPU from the amdgpu hwmon node (microwatts), sampled by a
    thread every 20 ms while a region runs."""

    def __init__(self):
        nodes = sorted(glob.glob("/sys/class/drm/card[0-9]*/device/hwmon/hwmon*/power1_input"))
        self.path = nodes[0] if nodes else None
        self.cap_w = None
        if self.path:
            try:
                self.cap_w = int(open(os.path.join(os.path.dirname(self.path), "power1_cap")).read()) / 1e6
            except (OSError, ValueError):
                pass
        self.samples = []
        self._stop = False
        self._thread = None

    def _run(self):
        while not self._stop:
            try:
                self.samples.append(int(open(self.path).read()) / 1e6)
            except (OSError, ValueError):
                pass
            time.sleep(0.02)

    def __enter__(self):
        if self.path:
            self._thread = threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        if self._thread:
            self._thread.join()

    def summary(self, skip_s=0.3):
        """Mean / max over the region without its first `skip_s` seconds (ramp-up)."""
        s = self.samples[int(skip_s / 0.02):] or self.samples
        if not s:
            return None
        return {"mean_w": sum(s) / len(s), "max_w": max(s), "cap_w": self.cap_w, "samples": len(s)}


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


def upload(w):
    import numpy as np
    import torch

    import workloads
    if w.dtype == "bf16":
        up = lambda a: torch.from_numpy(workloads.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        up = lambda a: torch.from_numpy(a).cuda()
    return up(w.X), up(w.W), torch.from_numpy(w.targets).cuda(), up


def time_steps(step, warmup, steps, with_power=False):
    """`steps` calls of step() after `warmup` untimed ones, bracketed by device
    synchronisation; returns (ms per step, sorted per-step ms from events on the call's
    stream, power summary or None)."""
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    sampler = PowerSampler() if with_power else None
    if sampler:
        sampler.__enter__()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    marks[0].record()
    for k in range(steps):
        step()
        marks[k + 1].record()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    if sampler:
        sampler.__exit__()
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
    # a region shorter than the ramp-up skip would leave nothing: skip less then
    power = sampler.summary(skip_s=min(0.3, (t2 - t1) / 4)) if sampler else None
    return (t2 - t1) * 1e3 / steps, per_step, power


def config_line(flce, w, code, ms, compaction, nh=1, flop_factor=6.0):
    """Throughput figures of one timed configuration."""
    rows = w.n_valid if compaction else w.BT
    nominal = flop_factor * w.BT * w.H * w.V * nh / (ms * 1e-3) / 1e12
    return {"ms_per_step": ms, "tokens_per_s": w.BT / (ms * 1e-3),
            "tflops_executed": nominal * rows / w.BT, "tflops_over_6BTHV": nominal,
            "rows_projected": rows, "row_compaction": bool(compaction),
            "chunks": flce.flce_num_chunks(w.BT, w.H, w.V, code),
            "chunk_rows": flce.flce_chunk_rows(w.BT, w.H, w.V, code),
            "peak_extra_hbm_mb": flce.flce_workspace_bytes(w.BT, w.H, w.V, code) / 1e6,
            "full_logits_avoided_mb": flce.flce_full_logits_bytes(w.BT, w.V, code) / 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
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
                    help="project every row, also those with an ignored target, in the headline leg too")
    ap.add_argument("--rmsnorm", action="store_true",
                    help="time flce_rmsnorm_fwd_bwd: RMSNorm of raw hidden states fused in front (one head)")
    ap.add_argument("--no-mfma-loop", action="store_true",
                    help="skip the MFMA-only loop that is reported beside the roofline")
    ap.add_argument("--mfma-loop-launches", type=int, default=160,
                    help="launches per operand pattern of the MFMA-only loop (about 2 ms each; the socket "
                         "power sensor needs a few seconds to settle)")
    ap.add_argument("--no-dense-leg", action="store_true", help="skip the leg with row compaction off")
    ap.add_argument("--no-per-config", action="store_true", help="skip the passes over the other four workloads")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one plain 1 GiB device copy first (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path is a single-GPU kernel "
              "pipeline; no collectives are part of it). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

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
    X, W, t, up = upload(w)
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
    variant = nh > 1 or args.rmsnorm or args.skip_dx
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

    # ---- headline leg: per-kernel timing off ----
    ms_per_step, per_step, power = time_steps(step, args.warmup, args.steps, with_power=True)
    quantile = lambda q: per_step[int(round(q * (len(per_step) - 1)))]
    loss_value = float(loss.item())
    tokens_per_s = w.BT / (ms_per_step * 1e-3)
    flop_factor = 4.0 if args.skip_dx else 6.0
    flops_step = flop_factor * w.BT * w.H * w.V * nh
    tflops_nominal = flops_step / (ms_per_step * 1e-3) / 1e12
    tflops_executed = tflops_nominal * rows_projected / (w.BT * nh)
    peak = MFMA_PEAK_TFLOPS[w.dtype]

    # ---- breakdown leg: the same passes with HIP events around every kernel launch ----
    # (two untimed passes are queued first and the switch is flipped while they run: a launch
    # that follows an idle GPU, even 15 ms of it, runs 10-18 % longer while the clock comes back)
    bsteps = max(1, min(args.steps, 5))
    for _ in range(2):
        step()
    flce.flce_timing_enable(True)
    for _ in range(bsteps):
        step()
    torch.cuda.synchronize()
    flce.flce_timing_enable(False)
    kt = flce.flce_timing_collect()
    nchunks = flce.flce_num_chunks(w.BT, w.H, w.V, code)
    gemm_kinds = ("logits_gemm", "dw_gemm") if args.skip_dx else ("logits_gemm", "dx_gemm", "dw_gemm")
    traffic = measured_traffic_bytes() if (args.config == 3 and not variant and not args.budget_mib
                                           and compaction) else {}
    # One product launch per chunk, head and class (the K-range reduction of a cut dX product is
    # booked with it).  Executed flops of a class per step: 2 * rows projected * H * V.
    # (with row compaction only the last ceil(N_valid / C) chunk launches of a head do any work)
    chunk_rows = flce.flce_chunk_rows(w.BT, w.H, w.V, code)
    if compaction:
        launches_per_step = sum(max(1, -(-int((x != w.ignore_index).sum().item()) // chunk_rows))
                                for x in all_targets)
    else:
        launches_per_step = nchunks * nh
    class_flops_step = 2.0 * rows_projected * w.H * w.V
    rooflines = {}
    for k in gemm_kinds:
        ms_step = kt[k][0] / bsteps
        avg_launch_ms = ms_step / launches_per_step
        ach = class_flops_step / launches_per_step / (avg_launch_ms * 1e-3) / 1e12 if ms_step > 0 else 0.0
        short = {"logits_gemm": "logits", "dx_gemm": "dx", "dw_gemm": "dw"}[k]
        rooflines[short] = {"bound": "mfma", "kernel": k, "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                            "frac": ach / peak, "ms_per_step": ms_step, "avg_launch_ms": avg_launch_ms,
                            "launches_per_step": launches_per_step,
                            "flops_per_launch": class_flops_step / launches_per_step,
                            "traffic": traffic.get(short)}
    dom = max(rooflines, key=lambda s: rooflines[s]["ms_per_step"])
    ce_ms, ce_n = kt["ce_rows"]
    elem = 2 if w.dtype == "bf16" else 4
    ce_gbs = (2.0 * rows_projected * w.V * elem * bsteps) / (ce_ms * 1e-3) / 1e9 if ce_n else 0.0

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
        # rows with an ignored target are left out of the products (row compaction): the matrix
        # cores execute 6 * rows_projected * H * V flops, not the nominal 6 * BT * H * V
        "row_compaction": bool(compaction),
        "rows_projected": rows_projected,
        "tflops_executed": tflops_executed,
        "mfma_util_frac_of_peak": tflops_executed / peak,
        "tflops_over_6BTHV": tflops_nominal,
        "mfma_util_frac_of_peak_nominal": tflops_nominal / peak,
        "peak_extra_hbm_mb": (flce.flce_rmsnorm_workspace_bytes if args.rmsnorm else
                              flce.flce_workspace_bytes)(w.BT, w.H, w.V, code) / 1e6,
        "full_logits_avoided_mb": flce.flce_full_logits_bytes(w.BT, w.V, code) / 1e6,
        "loss": loss_value,
        "socket_power": power,
        "kernel_ms_per_step": {k: kt[k][0] / bsteps for k in kt},
        "kernel_timing_steps": bsteps,
        "ce_rows_hbm_gbs": ce_gbs,
        "roofline": dict(rooflines[dom], dominant_of=sorted(rooflines)),
        "product_rooflines": rooflines,
    }

    # memory: the workspace is bounded whatever BT is; the logits it stands in for grow with BT
    out["memory"] = [{"BT": bt, "peak_extra_hbm_mb": flce.flce_workspace_bytes(bt, w.H, w.V, code) / 1e6,
                      "full_logits_avoided_mb": flce.flce_full_logits_bytes(bt, w.V, code) / 1e6,
                      "chunks": flce.flce_num_chunks(bt, w.H, w.V, code)}
                     for bt in (w.BT, 4 * w.BT, 16 * w.BT)]
    out["memory_bound_any_BT_mb"] = flce.flce_workspace_bytes_max(w.H, w.V, code) / 1e6
    # smallest BT (in steps of 256 rows) from which the workspace is smaller than the logits it
    # stands in for: below it the whole logits simply fit and the method has nothing to save
    bt = 256
    while flce.flce_workspace_bytes(bt, w.H, w.V, code) >= flce.flce_full_logits_bytes(bt, w.V, code) and bt < (1 << 24):
        bt += 256
    out["memory_break_even_BT"] = bt

    # ---- dense leg: every row projected, as the paper does ----
    if compaction and not args.no_dense_leg:
        flce.flce_set_row_compaction(False)
        try:
            dsteps = max(bsteps, min(args.steps, 15))
            dms, _, _ = time_steps(step, 2, dsteps)
        finally:
            flce.flce_set_row_compaction(True)
        dn = flops_step / (dms * 1e-3) / 1e12
        out["dense"] = {"what": "row compaction off: all BT rows projected", "ms_per_step": dms,
                        "tokens_per_s": w.BT / (dms * 1e-3), "tflops_executed": dn,
                        "mfma_util_frac_of_peak": dn / peak, "steps": dsteps}

    if w.dtype == "bf16" and not args.no_mfma_loop:
        # What the matrix pipes sustain with nothing to feed them from memory: the same MFMA
        # instruction in a loop on register operands, one wavefront per SIMD, launches about
        # as long as a product launch.  On operands like the workload's (normal deviates,
        # 4 x 4 fragments per K sub-step) the chip clocks far lower than on zeros.
        scratch = torch.empty(256 * 256, dtype=torch.float32, device="cuda")

        def mfma_loop(pattern, launches=max(16, args.mfma_loop_launches)):
            # a train of launches back to back (about 0.4 s by default): the clock settles
            # within the first launches, which are left out
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            fl = 0.0
            with PowerSampler() as ps:
                for k in range(launches):
                    if k == 8:
                        e0.record()
                    one = flce.flce_mfma_ceiling_launch(pattern, 256, 8000, 0.02, scratch)
                    fl += one if k >= 8 else 0.0
                e1.record()
                e1.synchronize()
            return fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, ps.summary(skip_s=0.1)

        (rnd, rnd_p), (zero, zero_p) = mfma_loop(2), mfma_loop(0)
        out["mfma_only_loop"] = {
            "random_operands_tflops": rnd, "zero_operands_tflops": zero,
            "random_operands_power": rnd_p, "zero_operands_power": zero_p,
            "what": "v_mfma_f32_32x32x16_bf16 on register operands, no memory traffic, 256 workgroups x 4 "
                    f"wavefronts, {max(16, args.mfma_loop_launches) - 8} launches of ~2-3 ms back to back after 8 to settle the clock; "
                    "random = N(0,1) x N(0,0.02^2) fragments, 4 A x 4 B per 16 MFMAs"}
        for r in out["product_rooflines"].values():
            r["frac_of_mfma_only_loop_random"] = r["achieved"] / rnd if rnd > 0 else None
        out["roofline"]["frac_of_mfma_only_loop_random"] = out["roofline"]["achieved"] / rnd if rnd > 0 else None

    # ---- the other benchmark workloads, a few passes each ----
    if not args.no_per_config and not variant and not args.budget_mib and not args.no_compaction:
        per = {}
        head_line = config_line(flce, w, code, ms_per_step, compaction)
        head_line["steps"] = args.steps
        per[f"config{args.config}"] = dict(head_line, workload=w.name, dtype=w.dtype)
        del X, W, t, dX, dW
        for idx in (1, 2, 3, 4, 5):
            if idx == args.config:
                continue
            wi = workloads.make_config(idx)
            ci = flce.FLCE_BF16 if wi.dtype == "bf16" else flce.FLCE_F32
            Xi, Wi, ti, _ = upload(wi)
            dXi, dWi = torch.empty_like(Xi), torch.empty_like(Wi)

            def step_i():
                flce.flce_fwd_bwd(Xi, Wi, ti, wi.ignore_index, loss=loss, dX=dXi, dW=dWi)

            # long enough (about 0.3 s) for the clock to settle after the idle time of the upload
            est, _, _ = time_steps(step_i, 1, 2)
            n = int(min(200, max(bsteps, -(-300.0 // max(est, 1e-3)))))
            msi, _, _ = time_steps(step_i, max(2, n // 4), n)
            comp_i = flce.flce_get_row_compaction() and wi.dtype == "bf16" and wi.H % 64 == 0
            line = config_line(flce, wi, ci, msi, comp_i)
            if msi < 1.0:
                # launch-bound: the same call recorded once into a HIP graph and replayed
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    step_i()
                line["graph_replay_ms"], _, _ = time_steps(graph.replay, max(2, n // 4), n)
                del graph
            line.update(workload=wi.name, dtype=wi.dtype, steps=n, loss=float(loss.item()),
                        mfma_util_frac_of_peak=line["tflops_executed"] / MFMA_PEAK_TFLOPS[wi.dtype])
            per[f"config{idx}"] = line
            del Xi, Wi, ti, dXi, dWi
            torch.cuda.empty_cache()
        per[f"config{args.config}"]["mfma_util_frac_of_peak"] = tflops_executed / peak
        per[f"config{args.config}"]["loss"] = loss_value
        out["per_config"] = [per[k] | {"config": k} for k in sorted(per)]

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
