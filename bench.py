#!/usr/bin/env python3
"""Benchmark of the fused multi-LoRA layer (forward + backward) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config I] [--no-configs] [--no-cpu]

A step is one pass of the whole hot path -- multi_lora_fwd then multi_lora_bwd in fused mode --
over one synthetic batch that is already resident in HBM.  The default (headline) workload is the
largest single-GPU config, the Llama-70B MLP shape (config 5: 16 adapters x 2048 tokens, ranks 16..128,
W 8192 x 28672, bf16); configs 2, 3 and 4 are timed in the same run and reported with the same fields
under `configs`.  Prints one JSON line: whole-job tokens/s, ms per step, the roofline of the dominant kernel
(per-kernel times from HIP events recorded on the launch stream), the LoRA-only path against
the HBM roofline, and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E


def bench_block(args, np, torch, ml, wl) -> int:
    """One step = forward of the seven projections, backward of the seven (reverse order), grouped AdamW of every
    adapter of every projection.  The plans of projections 2..7 reuse the first plan's segmentation tables."""
    from paper_2604_05426_amd.harness import DeviceBlock
    _, _, _, ranks, lens, scales, seed, _ = wl.config_shape(1)
    T, N = sum(lens), len(ranks)
    shapes = wl.LLAMA8B_BLOCK
    # plan construction: the first plan builds the segmentation tables, the others reuse them
    torch.cuda.synchronize()
    off = [0]
    for t in lens:
        off.append(off[-1] + t)
    t0 = time.perf_counter()
    base = ml.Plan(ml.BF16, T, shapes[0][1], shapes[0][2], ranks, scales, off)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    likes = [ml.Plan.like(base, k, n) for _, k, n in shapes[1:]]
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    owns = [ml.Plan(ml.BF16, T, k, n, ranks, scales, off) for _, k, n in shapes[1:]]
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for pl in likes + owns + [base]:
        pl.destroy()

    blk = DeviceBlock.synthetic("bf16", shapes, ranks, lens, scales, seed=100)
    blk.init_adamw()
    K, W = args.steps, args.warmup
    step_no = [0]

    def step():
        step_no[0] += 1
        blk.step([(1e-4, 0.9, 0.999, 1e-8, 0.0, step_no[0])] * N)

    for _ in range(W):
        step()
    torch.cuda.synchronize()
    t_settle, extra = time.perf_counter(), 0
    while time.perf_counter() - t_settle < 0.2 and extra < 200:     # clocks settle under load (see main)
        step(); step()
        torch.cuda.synchronize()
        extra += 2
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(K):
        step()
    end.record()
    torch.cuda.synchronize()
    ms = start.elapsed_time(end) / K
    # launches per step, from one event-profiled step
    launches = {}
    for dl in blk.layers:
        dl.plan.profile_begin(64)
    step()
    torch.cuda.synchronize()
    per_layer = {}
    for dl in blk.layers:
        recs = dl.plan.profile_end(64)
        per_layer[dl.w.name] = {"k": dl.w.k, "n": dl.w.n, "launches": len(recs), "ms": float(sum(m for _, m in recs))}
        for kid, _ in recs:
            launches[ml.KERNEL_NAMES[kid]] = launches.get(ml.KERNEL_NAMES[kid], 0) + 1
    R1 = sum(t * r for t, r in zip(lens, ranks))
    flops = sum(4.0 * T * k * n + 6.0 * R1 * (k + n) for _, k, n in shapes)
    out = {
        "metric": "multi-LoRA Llama-3.1-8B block (7 projections) fwd+bwd+AdamW tokens/s", "value": T / (ms * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "warmup_clock_settle_steps": extra, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama8b_block: q,k,v,o,gate,up,down over config 2's segmentation", "T": T, "adapters": N,
                   "ranks": ranks, "tokens_per_adapter": lens, "mode": "fused fwd+bwd per projection, grouped AdamW"},
        "tflops": flops / (ms * 1e-3) / 1e12,
        "frac_bf16_mfma_peak_whole_step": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "launches_per_step": launches, "launches_per_step_total": sum(launches.values()),
        "per_projection": per_layer,
        "plan_build_ms": {"first_plan": (t1 - t0) * 1e3, "six_more_sharing_its_tables": (t2 - t1) * 1e3,
                          "six_more_built_independently": (t3 - t2) * 1e3},
    }
    print(json.dumps(out))
    return 0


def bench_kernel_table(args, np, torch, ml, wl) -> int:
    """Grouped execution against launching the same kernels once per adapter, on the shape of the paper's kernel
    microbenchmark.  Ways to run one fwd+bwd of a 2048 x 2048 projection for 32 co-resident adapters:
      grouped      one plan over all adapters, fused step (this library's default);
      decoupled    one plan over all adapters, the paper's three-launch form: frozen-weight GEMMs (MLORA_FLAG_BASE_ONLY),
                   then grouped shrink and fused GEMM-add (MLORA_FLAG_LORA_ONLY);
      back_to_back the frozen-weight GEMMs once over the whole batch, then every adapter's LoRA terms on its own rows
                   through its own single-adapter plan, one after another;
      sequential   every adapter alone: its own fused step on its own rows, frozen-weight GEMM included.
    Every way is captured into a HIP graph once and the graph is replayed, so that what is compared is launches on the
    GPU and not the host's cost of issuing them (the eager, host-issued time of the grouped step is reported next to it)."""
    from paper_2604_05426_amd.harness import DeviceLayer
    k = n = 2048
    N, seq = 32, 256
    ranks = [[16, 32, 64][i % 3] for i in range(N)]
    scales = [2.0] * N            # alpha = 2r (the paper's training setting)
    K, W = args.steps, args.warmup
    rows = []

    def timed(fn):
        for _ in range(W):
            fn()
        torch.cuda.synchronize()
        t_settle = time.perf_counter()
        while time.perf_counter() - t_settle < 0.1:
            fn()
            torch.cuda.synchronize()
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        for _ in range(K):
            fn()
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) / K

    for bs in (1, 2, 4):
        lens = [bs * seq] * N
        dl = DeviceLayer.synthetic(f"bs{bs}", "bf16", k, n, ranks, lens, scales, seed=200 + bs)
        off = dl.w.offsets
        singles = []
        for i in range(N):
            pl = ml.Plan(ml.BF16, lens[i], k, n, [ranks[i]], [scales[i]], [0, lens[i]], stream=dl.stream)
            ws = torch.zeros(max(pl.workspace_bytes(), 256), dtype=torch.uint8, device=dl.device)
            Si = torch.zeros(max(lens[i] * ranks[i], 1), dtype=dl.tdtype, device=dl.device)
            singles.append((pl, ws, Si, slice(off[i], off[i + 1])))

        def grouped():
            dl.forward(); dl.backward()

        def decoupled():
            dl.forward(ml.FLAG_BASE_ONLY); dl.forward(ml.FLAG_LORA_ONLY)
            dl.backward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_LORA_ONLY)

        def per_adapter(flags):
            for i, (pl, ws, Si, sl) in enumerate(singles):
                ml.multi_lora_fwd(pl, dl.X[sl], dl.W, [dl.A[i]], [dl.B[i]], dl.Y[sl], Si, ws, flags, dl.stream)
                ml.multi_lora_bwd(pl, dl.dY[sl], dl.X[sl], dl.W, [dl.A[i]], [dl.B[i]], Si, dl.dX[sl], [dl.dA[i]], [dl.dB[i]],
                                  ws, flags, dl.stream)

        def back_to_back():
            dl.forward(ml.FLAG_BASE_ONLY); dl.backward(ml.FLAG_BASE_ONLY)
            per_adapter(ml.FLAG_LORA_ONLY)

        def sequential():
            per_adapter(0)

        def graphed(fn):
            fn()                                   # once eagerly: nothing is initialised inside the capture
            torch.cuda.synchronize()
            graph, side, eager_stream = torch.cuda.CUDAGraph(), torch.cuda.Stream(), dl.stream
            with torch.cuda.graph(graph, stream=side):
                dl.stream = torch.cuda.current_stream().cuda_stream
                fn()
            dl.stream = eager_stream
            return graph

        t_eager = timed(grouped)
        graphs = {name: graphed(fn) for name, fn in (("grouped", grouped), ("decoupled", decoupled),
                                                     ("back_to_back", back_to_back), ("sequential", sequential))}
        t = {name: timed(g.replay) for name, g in graphs.items()}
        rows.append({"per_adapter_batch": bs, "tokens": sum(lens), "grouped_eager_ms": t_eager, "grouped_ms": t["grouped"],
                     "decoupled_ms": t["decoupled"], "back_to_back_ms": t["back_to_back"], "sequential_ms": t["sequential"],
                     "decoupled_over_fused": t["decoupled"] / t["grouped"],
                     "grouped_over_back_to_back": t["back_to_back"] / t["grouped"],
                     "grouped_over_sequential": t["sequential"] / t["grouped"]})
        del graphs
        for pl, _, _, _ in singles:
            pl.destroy()
        dl.plan.destroy()
    out = {"metric": "grouped multi-LoRA layer fwd+bwd against per-adapter launches (speed-up)", "value": rows[0]["grouped_over_back_to_back"],
           "unit": "x", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": rows[0]["grouped_ms"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "kernel_table: 32 adapters, ranks 16/32/64 mixed, k = n = 2048, 256-token sequences", "adapters": N,
                      "ranks": ranks, "mode": "every variant replayed from a captured HIP graph"}, "table": rows}
    print(json.dumps(out))
    return 0


def bench_power_clock(args, np, torch, ml, wl) -> int:
    """Evidence for what bounds the frozen-weight GEMM: socket power and shader clock (sampled with amd-smi from a
    side thread) while, one after the other, the GPU idles, runs the register-only MFMA loop on zeros and on random
    operands, and runs the fused GEMMs of a config back to back; next to them the rates reached in the same run."""
    import re
    import subprocess
    import threading
    from paper_2604_05426_amd.harness import DeviceLayer
    cfg = args.config if args.config is not None else HEADLINE_CONFIG
    dtype, k, n, ranks, lens, scales, seed, _ = wl.config_shape(cfg - 1)
    dl = DeviceLayer.synthetic(f"config{cfg}", dtype, k, n, ranks, lens, scales, seed)
    T = dl.w.T
    scratch = torch.zeros(4096, dtype=torch.uint8, device=dl.device)

    def run_tool(cmd):
        try:
            return subprocess.run(cmd, capture_output=True, text=True, timeout=20).stdout
        except Exception:             # the tools are not part of the measurement: without them the fields stay empty
            return ""

    m = re.search(r"Max Graphics Package Power \(W\): ([0-9.]+)", run_tool(["rocm-smi", "--showmaxpower"]))
    power_limit = float(m.group(1)) if m else None

    def smi_sample():
        txt = run_tool(["amd-smi", "metric", "-p", "-c"])
        out = {}
        m = re.search(r"SOCKET_POWER: ([0-9.]+) W", txt)
        if m:
            out["power_w"] = float(m.group(1))
        clks = [float(x) for x in re.findall(r"GFX_\d+:\s+CLK: ([0-9.]+) MHz", txt)]     # one shader clock per XCD
        if clks:
            out["sclk_mhz"] = float(np.mean(clks))
        return out

    def phase(label, work, seconds):
        """Run `work` repeatedly for `seconds` while a side thread samples power and clock."""
        samples, stop = [], threading.Event()

        def sampler():
            time.sleep(0.3)           # let the phase reach its steady state
            while not stop.is_set():
                samples.append(smi_sample())

        th = threading.Thread(target=sampler)
        th.start()
        t0, reps = time.perf_counter(), 0
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        start.record()
        while time.perf_counter() - t0 < seconds:
            if work is None:
                time.sleep(0.05)
            else:
                for _ in range(4):
                    work()
                    reps += 1
                torch.cuda.synchronize()
        end.record()
        torch.cuda.synchronize()
        stop.set()
        th.join()
        pw = [x["power_w"] for x in samples if "power_w" in x]
        ck = [x["sclk_mhz"] for x in samples if "sclk_mhz" in x]
        return {"phase": label, "samples": len(samples), "power_w_mean": float(np.mean(pw)) if pw else None,
                "power_w_max": float(np.max(pw)) if pw else None, "sclk_mhz_mean": float(np.mean(ck)) if ck else None,
                "sclk_mhz_min": float(np.min(ck)) if ck else None, "power_limit_w": power_limit,
                "ms_per_call": start.elapsed_time(end) / max(reps, 1), "calls": reps}

    rows = [phase("idle", None, 2.0)]
    zeros = {}
    rows.append(phase("mfma loop, zero operands", lambda: zeros.update(t=ml.multi_lora_calib_mfma(False, scratch, dl.stream)), 3.0))
    rows[-1]["tflops"] = zeros["t"]
    rnd = {}
    rows.append(phase("mfma loop, random operands", lambda: rnd.update(t=ml.multi_lora_calib_mfma(True, scratch, dl.stream)), 3.0))
    rows[-1]["tflops"] = rnd["t"]
    flop = 2.0 * T * k * n
    for label, fn in (("fused GEMM forward (frozen weight only), back to back", lambda: dl.forward(ml.FLAG_BASE_ONLY)),
                      ("fused GEMM backward (frozen weight only), back to back", lambda: dl.backward(ml.FLAG_BASE_ONLY)),
                      ("whole fused step", lambda: (dl.forward(), dl.backward()))):
        dl.forward(); dl.backward()
        rows.append(phase(label, fn, 4.0))
        if "step" not in label:
            rows[-1]["tflops"] = flop / (rows[-1]["ms_per_call"] * 1e-3) / 1e12
            rows[-1]["frac_bf16_mfma_peak"] = rows[-1]["tflops"] / PEAK_BF16_MFMA_TFLOPS
            rows[-1]["frac_of_mfma_loop_random"] = rows[-1]["tflops"] / rnd["t"]
    out = {"metric": "socket power and shader clock under the fused GEMM", "value": rows[3].get("tflops"), "unit": "TFLOP/s",
           "n_gpus": 1, "steps": rows[3]["calls"], "warmup": 0, "ms_per_step": rows[3]["ms_per_call"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"config{cfg}:{wl.CONFIG_NAMES[cfg - 1]}", "T": T, "k": k, "n": n,
                      "mode": "socket power and the mean shader clock of the 8 XCDs, sampled with amd-smi while the kernels run"},
           "nominal_clock_mhz_of_published_peak": 2400, "phases": rows}
    print(json.dumps(out))
    return 0


KERNEL_SOURCES = ("mfma_common.h", "mfma_gemm.hip", "mfma_lora.hip", "plan.hip", "common.h")


def kernel_sources_sha256() -> str:
    """Hash of the kernel sources a PMC summary under profiles/ was measured on (it names the same hash)."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_05426_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def committed_traffic(config: int):
    """HBM-side bytes per launch from the committed rocprofv3 --pmc summary of this config (FETCH_SIZE and WRITE_SIZE,
    each scaled by what the same counter reads for a plain copy of known size).  The summary names the hash of the
    kernel sources it was measured on; if the sources have changed since, nothing is reported."""
    prof = os.path.join(ROOT, "profiles", f"bench_config{config}_pmc_traffic.md")
    if not os.path.exists(prof):
        return {}, None
    names = {"fused_gemm_kernel<true>": "gemm_fwd", "fused_gemm_kernel<false>": "gemm_bwd",
             "shrink_tiled_kernel<true": "shrink", "shrink_tiled_kernel<false": "dshrink",
             "shrink_kernel<true": "shrink", "shrink_kernel<false": "dshrink", "wgrad_kernel": "wgrad"}
    traffic, sha = {}, None
    for line in open(prof):
        parts = line.split()
        if len(parts) == 3 and parts[0] == "traffic_bytes":
            for key, short in names.items():        # (the launches of one step's rank classes add up)
                if parts[1].startswith(key):
                    traffic[short] = traffic.get(short, 0.0) + float(parts[2])
                    break
        if len(parts) == 2 and parts[0] == "kernel_sources_sha256":
            sha = parts[1]
    if sha != kernel_sources_sha256():
        return {}, f"profiles/{os.path.basename(prof)} was measured on other kernel sources"
    return traffic, f"profiles/{os.path.basename(prof)}"


def cpu_oracle_baseline(w, np, budget_s: float):
    """The CPU oracle as it stands (naive fp64 loops, OpenMP over rows) on a bounded sample of the workload: the first
    rows of every adapter's segment, whole fwd + bwd.  A short calibration run sizes the sample for about budget_s."""
    from oracle import multilora_oracle as orc

    def sample(per_adapter):
        keep, lens = [], []
        for i in range(w.N):
            c = min(per_adapter, w.seg_lens[i])
            keep.extend(range(w.offsets[i], w.offsets[i] + c))
            lens.append(c)
        off = [0] + [int(x) for x in np.cumsum(lens)]
        Xs, dYs = np.ascontiguousarray(w.X[keep]), np.ascontiguousarray(w.dY[keep])
        t0 = time.perf_counter()
        fw = orc.forward(Xs, w.W, w.A, w.B, w.scales, off)
        orc.backward(dYs, Xs, w.W, w.A, w.B, w.scales, off, S=fw.S)
        return len(keep), time.perf_counter() - t0

    # calibration: about 4 GFLOP of oracle work, at least one token per adapter
    per_token = 4.0 * w.k * w.n
    cal_per_adapter = int(max(1, min(max(w.seg_lens), 4e9 / per_token / max(1, w.N))))
    cal_tokens, cal_dt = sample(cal_per_adapter)
    # A call has a fixed cost (thread start, widening W to fp64) next to the cost per token: two small runs give both,
    # and the final sample is sized so that the whole call takes about budget_s.
    cap = max(w.seg_lens)
    mid_per_adapter = min(cap, max(cal_per_adapter + 1, 3 * cal_per_adapter))
    mid_tokens, mid_dt = sample(mid_per_adapter)
    if mid_tokens > cal_tokens and mid_dt > cal_dt:
        per_token = (mid_dt - cal_dt) / (mid_tokens - cal_tokens)
        fixed = max(0.0, cal_dt - per_token * cal_tokens)
    else:
        per_token, fixed = mid_dt / max(mid_tokens, 1), 0.0
    per_adapter = int(max(1, min(cap, (budget_s - fixed) / max(per_token, 1e-9) / max(1, w.N))))
    ntok, dt = sample(per_adapter)
    return {"value": ntok / dt, "unit": "tokens/s", "cores": orc.num_threads(), "kind": "oracle", "seconds": dt,
            "sample": f"first {per_adapter} tokens of each of the {w.N} adapters ({ntok} of {w.T} tokens), "
                      f"whole fwd+bwd (Y, S, dS, dX, dA_i, dB_i), naive fp64 loops"}


class PowerClockSampler:
    """Samples socket power and the mean shader clock of the XCDs with amd-smi from a side thread (about ten samples a
    second) while the main thread keeps the GPU busy.  Missing tool or unparsable output: no samples, fields stay None."""

    def __init__(self, np):
        import threading
        self.np, self.samples, self._stop = np, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        while not self._stop.is_set():
            try:
                txt = subprocess.run(["amd-smi", "metric", "-p", "-c"], capture_output=True, text=True, timeout=20).stdout
            except Exception:
                return
            m = re.search(r"SOCKET_POWER: ([0-9.]+) W", txt)
            clks = [float(x) for x in re.findall(r"GFX_\d+:\s+CLK: ([0-9.]+) MHz", txt)]
            if m and clks:
                self.samples.append((float(m.group(1)), float(self.np.mean(clks))))

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self):
        if not self.samples:
            return {"samples": 0, "socket_power_w_mean": None, "shader_clock_mhz_mean": None}
        pw, ck = [x[0] for x in self.samples], [x[1] for x in self.samples]
        return {"samples": len(pw), "socket_power_w_mean": float(self.np.mean(pw)), "socket_power_w_max": float(max(pw)),
                "shader_clock_mhz_mean": float(self.np.mean(ck)), "shader_clock_over_nominal_2400": float(self.np.mean(ck)) / 2400.0}


def measure_layer(config: int, args, mods, extras: bool, lora_and_base: bool, ceilings: bool, cpu_budget_s: float,
                  power: bool = False) -> dict:
    """Everything bench.py reports for one benchmark config (1-based): the timed fused step, per-kernel times and
    roofline fractions, the LoRA-only path against the HBM roofline, the frozen-weight GEMMs alone, the CPU oracle."""
    np, torch, ml, wl, DeviceLayer = mods
    t_draw = time.perf_counter()
    w = wl.config(config - 1)
    dl = DeviceLayer(w, canary=0.0, guards=False)
    draw_s = time.perf_counter() - t_draw
    K, W = args.steps, args.warmup
    T, k, n, R1 = w.T, w.k, w.n, w.R1
    e = 2 if w.dtype == "bf16" else 4
    sum_r = sum(r for r, t in zip(w.ranks, w.seg_lens) if t > 0)

    def step(flags=0):
        dl.forward(flags)
        dl.backward(flags)

    def timed(fn, reps):
        start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        start.record()
        for _ in range(reps):
            fn()
        end.record()
        torch.cuda.synchronize()
        return start.elapsed_time(end) / reps

    for _ in range(W):
        step()
    # The GPU's power management needs tens of milliseconds of continuous load to settle its clocks (the first ~50 steps
    # after idle run up to 10 % slower).  Keep stepping, untimed, until 0.2 s of load have passed, so that the K timed
    # steps measure the steady state whatever W was asked for.
    extra_warmup = 0
    torch.cuda.synchronize()
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.2 and extra_warmup < 2000:
        for _ in range(10 if T * k * n < 1e12 else 2):
            step()
            extra_warmup += 1
        torch.cuda.synchronize()
    ms_step = timed(step, K)

    flops_base = 4.0 * T * k * n
    flops_lora = 6.0 * R1 * (k + n)
    flops = flops_base + flops_lora
    out = {
        "workload": f"config{config}:{w.name}", "dtype": w.dtype, "T": T, "k": k, "n": n, "adapters": w.N,
        "ranks": w.ranks, "tokens_per_adapter": w.seg_lens, "mode": "fused fwd+bwd",
        "value": T / (ms_step * 1e-3), "unit": "tokens/s", "ms_per_step": ms_step, "steps": K, "warmup": W,
        "warmup_clock_settle_steps": extra_warmup,
        "tflops": flops / (ms_step * 1e-3) / 1e12,
        "frac_bf16_mfma_peak_whole_step": flops / (ms_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
        "host_input_generation_s": draw_s,
    }

    if extras:
        # per-kernel times: the same K steps again, every launch bracketed by HIP events on its stream
        dl.plan.profile_begin(K * 16)
        for _ in range(K):
            step()
        recs = dl.plan.profile_end(K * 16)
        per = {}
        for kid, ms in recs:
            per.setdefault(ml.KERNEL_NAMES[kid], []).append(ms)
        kern = {name: {"launches_per_step": len(v) / K, "avg_ms": float(np.mean(v))} for name, v in per.items()}
        # algorithmic work of one launch of each kernel
        alg = {
            "gemm_fwd": ("mfma", 2.0 * T * k * n + 2.0 * R1 * n),
            "gemm_bwd": ("mfma", 2.0 * T * k * n + 2.0 * R1 * k),
            "shrink": ("hbm", (T * k + sum_r * k + R1) * e),
            "dshrink": ("hbm", (T * n + sum_r * n + R1) * e),
            "wgrad": ("hbm", (T * k + T * n + 2 * R1 + sum_r * (k + n)) * e),
        }
        for name, (bound, work) in alg.items():
            if name in kern:
                # a kernel that a plan launches several times per step (one launch per rank class) is priced as a whole
                t = kern[name]["avg_ms"] * kern[name]["launches_per_step"] * 1e-3
                if bound == "mfma":
                    kern[name].update(bound="mfma", achieved_tflops=work / t / 1e12,
                                      frac=work / t / 1e12 / PEAK_BF16_MFMA_TFLOPS)
                else:
                    kern[name].update(bound="hbm", achieved_gbs=work / t / 1e9, frac=work / t / 1e9 / PEAK_HBM_GBS)
        out["kernels"] = kern
        # forward and backward by themselves: the sum of their launches' own durations (HIP events around every launch)
        fwd_names, tot = ("shrink", "gemm_fwd"), lambda nm: kern[nm]["avg_ms"] * kern[nm]["launches_per_step"]
        if all(nm in kern for nm in fwd_names):
            out["fwd_ms_kernels"] = float(sum(tot(nm) for nm in fwd_names))
            out["bwd_ms_kernels"] = float(sum(tot(nm) for nm in kern if nm not in fwd_names))
        traffic, traffic_source = committed_traffic(config)
        named = [nm for nm in kern if nm in alg]
        if not named:
            # fp32 / odd-width plans run every step through the grouped FMA kernel on the vector ALUs
            out["roofline"] = {"kernel": "fma_grouped_gemm_kernel (all launches of a step)", "bound": "alu",
                               "achieved": flops / (ms_step * 1e-3) / 1e12, "peak": 157.3, "unit": "TFLOP/s",
                               "frac": flops / (ms_step * 1e-3) / 1e12 / 157.3, "traffic": None}
        dom = max(named, key=lambda nm: kern[nm]["avg_ms"] * kern[nm]["launches_per_step"]) if named else None
        bound, work = alg[dom] if dom else (None, 0.0)
        t = kern[dom]["avg_ms"] * kern[dom]["launches_per_step"] * 1e-3 if dom else 1.0
        if bound == "mfma":
            out["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": work / t / 1e12, "peak": PEAK_BF16_MFMA_TFLOPS,
                               "unit": "TFLOP/s", "frac": work / t / 1e12 / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic.get(dom),
                               "traffic_source": traffic_source, "algorithmic_flop_per_launch": work,
                               "avg_kernel_ms": kern[dom]["avg_ms"]}
        elif bound == "hbm":
            out["roofline"] = {"kernel": dom, "bound": "hbm", "achieved": work / t / 1e9, "peak": PEAK_HBM_GBS,
                               "unit": "GB/s", "frac": work / t / 1e9 / PEAK_HBM_GBS, "traffic": traffic.get(dom),
                               "traffic_source": traffic_source, "algorithmic_bytes_per_launch": work,
                               "avg_kernel_ms": kern[dom]["avg_ms"]}
        if traffic:
            out["traffic_per_launch_bytes"] = traffic

    if power:
        # socket power and shader clock while the fused step runs back to back for about two seconds (the published MFMA
        # peak assumes 2400 MHz; under this step the board sits at its power limit and clocks lower)
        with PowerClockSampler(np) as smp:
            t_end = time.perf_counter() + 2.0
            while time.perf_counter() < t_end:
                for _ in range(4):
                    step()
                torch.cuda.synchronize()
        out["power_clock_under_fused_step"] = smp.summary()

    if extras and lora_and_base:
        # LoRA grouped path alone (W skipped; Y and dX updated in place) against the HBM roofline
        for _ in range(2):
            step(ml.FLAG_LORA_ONLY)
        ms_lf = timed(lambda: dl.forward(ml.FLAG_LORA_ONLY), K)
        ms_lb = timed(lambda: dl.backward(ml.FLAG_LORA_ONLY), K)
        small = (2 * sum_r * (k + n) + 2 * R1) * e
        bytes_f = (T * k + 2 * T * n) * e + (sum_r * (k + n) + 2 * R1) * e
        bytes_b = (2 * T * n + T * k + 2 * T * k) * e + small + 3 * R1 * e
        # per-kernel times of the same path (expand-add launches report under the ids of the GEMMs they stand in for)
        dl.plan.profile_begin(K * 16)
        for _ in range(K):
            step(ml.FLAG_LORA_ONLY)
        per_lo = {}
        for kid, ms in dl.plan.profile_end(K * 16):
            per_lo.setdefault({"gemm_fwd": "expand_add_fwd", "gemm_bwd": "expand_add_bwd"}.get(ml.KERNEL_NAMES[kid], ml.KERNEL_NAMES[kid]), []).append(ms)
        alg_lo = {"shrink": (T * k + sum_r * k + R1) * e, "dshrink": (T * n + sum_r * n + R1) * e,
                  "wgrad": (T * k + T * n + 2 * R1 + sum_r * (k + n)) * e,
                  "expand_add_fwd": (2 * T * n + R1 + sum_r * n) * e, "expand_add_bwd": (2 * T * k + R1 + sum_r * k) * e}
        kern_lo = {}
        for name, v in per_lo.items():
            t = float(np.sum(v)) / K * 1e-3
            kern_lo[name] = {"ms_per_step": t * 1e3}
            if name in alg_lo:
                kern_lo[name].update(algorithmic_bytes=alg_lo[name], achieved_gbs=alg_lo[name] / t / 1e9, frac_hbm=alg_lo[name] / t / 1e9 / PEAK_HBM_GBS)
        out["lora_path"] = {
            "mode": "MLORA_FLAG_LORA_ONLY", "fwd_ms": ms_lf, "bwd_ms": ms_lb, "kernels": kern_lo,
            "fwd_gbs": bytes_f / (ms_lf * 1e-3) / 1e9, "bwd_gbs": bytes_b / (ms_lb * 1e-3) / 1e9,
            "frac_hbm": (bytes_f + bytes_b) / ((ms_lf + ms_lb) * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "algorithmic_bytes_fwd": bytes_f, "algorithmic_bytes_bwd": bytes_b,
        }
        # frozen-weight GEMMs alone, for the cost of the LoRA terms inside the fused step
        for _ in range(2):
            step(ml.FLAG_BASE_ONLY)
        ms_base = timed(lambda: step(ml.FLAG_BASE_ONLY), K)
        # the paper's decoupled execution (base GEMM, grouped shrink, fused GEMM-add as separate launches) is
        # BASE_ONLY followed by LORA_ONLY; the default fused step folds the expand into the base GEMM
        out["decoupled"] = {"ms_per_step": ms_base + ms_lf + ms_lb, "decoupled_over_fused": (ms_base + ms_lf + ms_lb) / ms_step}
        out["base_only"] = {"ms_per_step": ms_base, "tflops": flops_base / (ms_base * 1e-3) / 1e12,
                            "frac_bf16_mfma_peak": flops_base / (ms_base * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS,
                            "fused_over_base": ms_step / ms_base}

    if ceilings:
        # what this GPU sustains right now for the two resources the fractions above are priced against (the published
        # peaks stay the denominators of `frac`): a register-only loop of the GEMM's 16x16x32 MFMAs on random operands
        # (runs into the board power limit like the GEMM does) and on zeros (no throttling), and a streaming read
        scratch = torch.zeros(4096, dtype=torch.uint8, device=dl.device)
        buf = torch.zeros(1 << 30, dtype=torch.uint8, device=dl.device)
        meas = {
            "mfma_loop_random_tflops": ml.multi_lora_calib_mfma(True, scratch, dl.stream),
            "mfma_loop_zeros_tflops": ml.multi_lora_calib_mfma(False, scratch, dl.stream),
            "stream_read_gbs": ml.multi_lora_calib_read(buf, 1 << 30, scratch, dl.stream),
        }
        del buf
        out["measured_ceilings"] = meas
        if out.get("roofline", {}).get("bound") == "mfma":
            out["roofline"]["frac_of_measured_mfma_loop"] = out["roofline"]["achieved"] / meas["mfma_loop_random_tflops"]
        if "lora_path" in out:
            lp = out["lora_path"]
            lp["frac_of_measured_stream_read"] = ((lp["fwd_gbs"] * lp["fwd_ms"] + lp["bwd_gbs"] * lp["bwd_ms"])
                                                  / (lp["fwd_ms"] + lp["bwd_ms"]) / meas["stream_read_gbs"])

    if args.calib_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dl.device)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calib_copy_bytes"] = 1 << 30
        del src, dst

    dl.plan.destroy()
    del dl
    torch.cuda.empty_cache()
    if cpu_budget_s > 0:
        out["cpu_baseline"] = cpu_oracle_baseline(w, np, cpu_budget_s)
    return out


HEADLINE_CONFIG = 5       # the largest single-GPU configuration: Llama-70B MLP shape, 16 adapters x 2048 tokens
OTHER_CONFIGS = (2, 3, 4)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="time only this benchmark config (1..5).  Default: config 5 (Llama-70B MLP shape) as the headline, "
                         "and configs 2, 3, 4 with the same fields in `configs`")
    ap.add_argument("--no-configs", action="store_true", help="headline config only, no `configs` array")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-kernel / LoRA-only passes")
    ap.add_argument("--fused-only", action="store_true",
                    help="skip the LoRA-only and base-only passes (every launch is then the fused-mode one; used under rocprofv3)")
    ap.add_argument("--block", action="store_true",
                    help="time a whole LoRA'd Llama-3.1-8B block instead of one layer: the seven projections over one "
                         "segmentation (config 2's adapters), fwd, bwd and the grouped AdamW update")
    ap.add_argument("--kernel-table", action="store_true",
                    help="the paper's kernel microbenchmark shape (Sec. 8.3 ablation, kernel table): 32 adapters, ranks "
                         "16/32/64 equally mixed, Llama-3.2-1B width, per-adapter batch 1/2/4 x 256 tokens; grouped launch "
                         "against per-adapter launches of the same kernels")
    ap.add_argument("--power-clock", action="store_true",
                    help="sample socket power and shader clock (amd-smi) while the MFMA calibration loops and the fused GEMMs "
                         "of --config (default: the headline config) run: the evidence for what bounds the GEMM")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1. Adapters would shard across GPUs as disjoint row segments.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_05426_amd import binding as ml
    from paper_2604_05426_amd import workloads as wl
    from paper_2604_05426_amd.harness import DeviceLayer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    ml.lib()   # fail loudly if the extension is missing

    if args.block:
        return bench_block(args, np, torch, ml, wl)
    if args.kernel_table:
        return bench_kernel_table(args, np, torch, ml, wl)
    if args.power_clock:
        return bench_power_clock(args, np, torch, ml, wl)

    mods = (np, torch, ml, wl, DeviceLayer)
    head_cfg = args.config if args.config is not None else HEADLINE_CONFIG
    extras = not args.no_extra
    full = extras and not args.fused_only
    h = measure_layer(head_cfg, args, mods, extras=extras, lora_and_base=full, ceilings=full,
                      cpu_budget_s=0.0 if args.no_cpu else 12.0, power=full)
    out = {
        "metric": "multi-LoRA layer fwd+bwd tokens/s", "value": h["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": h["steps"], "warmup": h["warmup"], "warmup_clock_settle_steps": h["warmup_clock_settle_steps"],
        "ms_per_step": h["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": h["dtype"], "data": "synthetic",
        "config": {"workload": h["workload"], "T": h["T"], "k": h["k"], "n": h["n"], "adapters": h["adapters"],
                   "ranks": h["ranks"], "tokens_per_adapter": h["tokens_per_adapter"], "mode": h["mode"]},
    }
    for key in ("tflops", "frac_bf16_mfma_peak_whole_step", "fwd_ms_kernels", "bwd_ms_kernels", "kernels", "roofline", "traffic_per_launch_bytes", "lora_path",
                "decoupled", "base_only", "measured_ceilings", "power_clock_under_fused_step", "calib_copy_bytes", "cpu_baseline",
                "host_input_generation_s"):
        if key in h:
            out[key] = h[key]
    if args.config is None and not args.no_configs:
        # the other bf16 configs, same fields, a shorter CPU leg each
        out["configs"] = [measure_layer(c, args, mods, extras=extras, lora_and_base=full, ceilings=False,
                                        cpu_budget_s=0.0 if args.no_cpu else 3.0) for c in OTHER_CONFIGS]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
