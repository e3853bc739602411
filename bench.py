#!/usr/bin/env python3
"""Benchmark of the CoPRIS rollout-decode hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input:
  copris_decode_attn (split-K attention + merge: one layer's KV) +
  copris_lmhead_logprob (LM head + log-softmax + Gumbel-max + log-prob gather)
on the 7B-shaped C=256 decode configuration, + copris_is_ratio on the cross-stage IS
batch (256 trajectories).  All inputs are resident in HBM before the timed region.

Protocol: W untimed warm-up steps, then exactly K steps timed by wall clock between two
device synchronisations (`value`, `ms_per_step`); inside the same K steps an event pair
around every call gives per-call medians with p10 / p90; a second, instrumented pass of K
steps (the library's launch hook records an event before and after every kernel launch on
the launching stream) gives per-kernel durations.  Workloads smaller than the 256 MB
Infinity Cache (the IS batch, the 1.5B-shaped step) rotate over physically distinct input
sets so that repeats are served by HBM, not by the cache.

Prints ONE JSON line: decode tokens/s (C / step time), the HBM roofline of both main
kernels (algorithmic bytes / kernel duration vs 8 TB/s; `roofline` is the one further from
its roof), the practical ceilings measured in the same run (a plain 1 GiB device copy, the
core clock under the LM-head kernel on the seeded operands and on zeros) and the fp64 CPU
oracle timed on the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published
CACHE_ROTATION_SETS = 8         # distinct input sets for cache-sized workloads
SETTLE_STEPS = 50      # untimed steps before the timed region (warm-up steps count towards them)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, choices=[0, 1, 2],
                    help="decode config index (2 = the 7B-shaped C=256 config the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=256, help="sequences in the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run the plain 1 GiB device copy right after the warm-up as well (known traffic: "
                         "the scale for the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--token-logprob-m", type=int, default=8192,
                    help="positions in the micro-batch of the given-token log-prob measurement")
    ap.add_argument("--no-extras", action="store_true", help="time the step only")
    ap.add_argument("--no-longtail", action="store_true",
                    help="skip the decode-attention measurement on the long-tail stress configuration")
    ap.add_argument("--prefill-seqs", type=int, default=16,
                    help="resumed trajectories in the re-prefill attention measurement")
    ap.add_argument("--lib", default=None, help="path of a libcopris build to measure instead of the in-tree one")
    return ap.parse_args()


def algorithmic_bytes(cfg, inp, isb):
    """Bytes the method itself must move, per launch: K and V rows of every context token, the
    block-table entries used, q in and out; W once plus hidden and the per-row outputs; 17 bytes
    per token of the ratio batch."""
    import numpy as np
    eb = cfg.elem_bytes
    ctx = inp["ctx_len"].astype(np.int64)
    pages = (ctx + cfg.page_size - 1) // cfg.page_size
    kv = int(ctx.sum()) * 2 * cfg.Hkv * cfg.D * eb            # K and V rows of every context token
    attn = kv + int(pages.sum()) * 4 + 2 * cfg.C * cfg.Hq * cfg.D * eb   # + block table + q in + out
    lm = cfg.V * cfg.H * eb + cfg.C * cfg.H * eb + 12 * cfg.C  # W once + hidden + token/logprob/lse
    is_ = 17 * int(isb["N"]) if isb is not None else 0          # cur + selected old + mask in, 2 outputs
    return {"attn": attn, "lm": lm, "is": is_, "kv": kv}


def dist(samples):
    """median / p10 / p90 / mean of a list of milliseconds."""
    import numpy as np
    a = np.asarray(samples, dtype=np.float64)
    return {"median": round(float(np.median(a)), 4), "p10": round(float(np.percentile(a, 10)), 4),
            "p90": round(float(np.percentile(a, 90)), 4), "mean": round(float(a.mean()), 4), "n": int(a.size)}


def time_rotating(runs, stream, n, warmup):
    """Event-timed calls, call i using runs[i % len(runs)]; returns the list of milliseconds."""
    import torch
    for i in range(warmup):
        runs[i % len(runs)]()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i, (a, b) in enumerate(ev):
        a.record(stream)
        runs[i % len(runs)]()
        b.record(stream)
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


class ClockSampler:
    """Samples the GPU core clock the driver reports (the starred level of pp_dpm_sclk) and the
    board power (hwmon power1_input) from a host thread while a kernel loop runs."""

    def __init__(self):
        paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.path = paths[0] if paths else None
        hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.power_path = hw[0] if hw else None
        self.samples = []
        self.power = []
        self.last_power_w = None
        self._stop = threading.Event()

    def power_cap_w(self):
        try:
            return round(float(open(self.power_path.replace("power1_input", "power1_cap")).read()) * 1e-6, 1)
        except Exception:
            return None

    def _read_power(self):
        try:
            return float(open(self.power_path).read()) * 1e-6
        except Exception:
            return None

    def _read(self):
        try:
            for line in open(self.path).read().splitlines():
                if line.rstrip().endswith("*"):
                    return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except Exception:
            return None
        return None

    def _loop(self):
        while not self._stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            w = self._read_power() if self.power_path else None
            if w is not None:
                self.power.append(w)
            time.sleep(0.005)

    def measure(self, fn, seconds):
        """Runs fn() back to back for about `seconds`; returns the median sampled clock in MHz
        (None if the driver file is not readable) and the mean milliseconds per call."""
        import numpy as np
        import torch
        if self.path is None:
            return None, None
        self.samples = []
        self.power = []
        self._stop.clear()
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        th = threading.Thread(target=self._loop, daemon=True)
        calls = 0
        t0 = time.perf_counter()
        th.start()
        while time.perf_counter() - t0 < seconds:
            for _ in range(50):
                fn()
            torch.cuda.synchronize()
            calls += 50
        dt = time.perf_counter() - t0
        self._stop.set()
        th.join()
        body = self.samples[len(self.samples) // 4:]        # the ramp-up is not the sustained state
        pw = self.power[len(self.power) // 4:]
        self.last_power_w = round(float(np.median(pw)), 1) if pw else None
        return (round(float(np.median(body)), 1) if body else None), round(dt * 1e3 / calls, 4)


def cpu_baseline(cfg, inp, n_sample):
    """The fp64 oracle, as it stands, on the first n_sample sequences of the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import copris_oracle as O
    from paper_2511_05589_amd import workloads as W

    seqs = np.arange(min(n_sample, cfg.C))
    P = cfg.page_size
    npg = (inp["ctx_len"][seqs].astype(np.int64) + P - 1) // P
    pages = np.concatenate([inp["block_table"][s, :n] for s, n in zip(seqs, npg)])
    bt = np.full((len(seqs), int(npg.max())), -1, dtype=np.int32)
    off = 0
    for i, n in enumerate(npg):
        bt[i, :n] = np.arange(off, off + n)
        off += n
    f = lambda a: W.to_f32(a, cfg.dtype)
    q, kc, vc = f(inp["q"][seqs]), f(inp["k_cache"][pages]), f(inp["v_cache"][pages])
    hid, wt = f(inp["hidden"][seqs]), f(inp["weight"])
    # whole passes over the sample until about 10 s of CPU work have been timed
    t_attn = t_lm = 0.0
    passes = 0
    while passes == 0 or (t_attn + t_lm < 10.0 and passes < 20):
        t0 = time.perf_counter()
        O.decode_attn(q, kc, vc, bt, inp["ctx_len"][seqs], inp["scale"])
        t1 = time.perf_counter()
        O.lmhead_logprob(hid, wt, inp["seq_id"][seqs], inp["step"][seqs], inp["seed"], inp["temperature"])
        t2 = time.perf_counter()
        t_attn += t1 - t0
        t_lm += t2 - t1
        passes += 1
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    total = t_attn + t_lm
    return {"value": round(len(seqs) * passes / total, 2), "unit": "tokens/s", "cores": int(threads),
            "kind": "oracle",
            "sample": (f"first {len(seqs)} of {cfg.C} sequences of the same workload, {passes} pass(es): "
                       f"oracle attention over their full contexts ({t_attn / passes:.2f} s/pass) + oracle LM "
                       f"head / sampling for their rows incl. widening W to fp64 ({t_lm / passes:.2f} s/pass); "
                       f"numpy fp64, BLAS threads {threads}, {len(os.sched_getaffinity(0))} cores visible"),
            "seconds": round(total, 3)}


def clone_device(d):
    """A physically distinct copy of a staged call (every tensor field cloned)."""
    import dataclasses
    import torch
    return dataclasses.replace(d, **{f.name: getattr(d, f.name).clone() for f in dataclasses.fields(d)
                                     if isinstance(getattr(d, f.name), torch.Tensor)})


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_05589_amd import binding, runner, workloads as W

    if args.lib:
        binding.load_library(os.path.abspath(args.lib))
    dev = runner.require_gpu()
    cfg = W.DECODE_CONFIGS[args.config]
    t_gen = time.perf_counter()
    inp = W.make_decode_inputs(cfg)
    isb = W.make_is_inputs(W.IS_CONFIGS[4 if args.config != 0 else 0])
    t_gen = time.perf_counter() - t_gen

    attn = runner.stage_attn(inp, cfg.dtype, dev)
    lm = runner.stage_lmhead(inp, cfg.dtype, dev)
    # the IS batch (47 MB with its outputs) would sit in the Infinity Cache: rotate over distinct copies
    isd = [runner.stage_is_ratio(isb, dev) for _ in range(CACHE_ROTATION_SETS)]
    stream = torch.cuda.current_stream()
    ab = algorithmic_bytes(cfg, inp, isb)

    def step(k):
        attn.run(stream)
        lm.run(stream)
        isd[k % len(isd)].run(stream)

    # The chip needs some tens of launches after staging to reach its sustained state (clocks
    # ramp up from idle; the LM-head kernel gets ~3 % faster over its first ~50 launches), so the
    # device is brought there first whatever W is; then the W warm-up steps of the contract.
    for k in range(max(0, SETTLE_STEPS - args.warmup)):
        step(k)
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()

    def device_copy_1gib():
        """Plain 1 GiB device copy (reads 1 GiB, writes 1 GiB); returns GB/s moved."""
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        dst.copy_(src)
        e1.record(stream)
        torch.cuda.synchronize()
        return 2.0 * (1 << 30) / (e0.elapsed_time(e1) * 1e-3) / 1e9

    if args.copy_calibration:
        device_copy_1gib()

    # ---- timed region: exactly K steps, events around each of the three calls ----
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record(stream)
        attn.run(stream)
        ev[k][1].record(stream)
        lm.run(stream)
        ev[k][2].record(stream)
        isd[k % len(isd)].run(stream)
        ev[k][3].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    call = {name: dist([ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(args.steps)])
            for i, name in enumerate(["attn", "lm", "is"])}
    call_ms = {k: v["median"] for k, v in call.items()}

    # ---- per-kernel durations: the library's launch hook records an event before and
    # after every kernel launch (same stream, same K steps, instrumented pass) ----
    recs = []
    # (events made beforehand: the hook must cost the host less than the kernels cost the GPU,
    # or the launches arrive late and every kernel starts on an idle chip)
    pool = [torch.cuda.Event(enable_timing=True) for _ in range(16 * args.steps + 64)]
    names = {}

    def hook(kernel, phase, _stream, _user):
        e = pool[len(recs)]
        e.record(stream)
        recs.append((names.setdefault(kernel, kernel.decode()), phase, e))

    for k in range(SETTLE_STEPS):          # (the chip idled while the host worked out the figures above)
        step(k)
    binding.set_launch_hook(hook)
    for k in range(args.steps):
        step(k)
    torch.cuda.synchronize()
    binding.set_launch_hook(None)
    per_kernel = {}
    for i in range(0, len(recs), 2):
        (name, p0, e0), (name1, p1, e1) = recs[i], recs[i + 1]
        assert name == name1 and p0 == 0 and p1 == 1
        per_kernel.setdefault(name, []).append(e0.elapsed_time(e1))
    kernel_dist = {k: dist(v) for k, v in per_kernel.items()}
    kernel_ms = {k: v["mean"] for k, v in kernel_dist.items()}      # average launch duration

    # ---- rooflines of the two main kernels (and the ratio kernel) ----
    main_kernels = {"attn": next(k for k in kernel_ms if k.startswith("attn_split")),
                    "lm": next(k for k in kernel_ms if k.startswith("lmhead") and "merge" not in k),
                    "is": "is_ratio_kernel"}
    traffic = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"config{args.config}", {})
    kernels = {}
    for part, kname in main_kernels.items():
        gbs = ab[part] / (kernel_ms[kname] * 1e-3) / 1e9
        kernels[kname] = {"avg_ms": round(kernel_ms[kname], 4), "median_ms": kernel_dist[kname]["median"],
                          "p10_ms": kernel_dist[kname]["p10"], "p90_ms": kernel_dist[kname]["p90"],
                          "algorithmic_bytes": ab[part], "achieved_GBps": round(gbs, 1),
                          "frac_hbm": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(kname)}
    lm_flops = 2.0 * cfg.C * cfg.H * cfg.V
    kernels[main_kernels["lm"]]["mfma_frac"] = round(
        lm_flops / (kernel_ms[main_kernels["lm"]] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)

    def roof(kname):
        return {"bound": "hbm", "kernel": kname, "achieved": kernels[kname]["achieved_GBps"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels[kname]["frac_hbm"],
                "traffic": kernels[kname]["traffic"], "avg_kernel_ms": kernels[kname]["avg_ms"]}

    two = [main_kernels["attn"], main_kernels["lm"]]
    low = min(two, key=lambda k: kernels[k]["frac_hbm"])      # the kernel further from its roof
    roofline = roof(low)
    roofline["other_main_kernel"] = roof([k for k in two if k != low][0])
    pair_ms = call_ms["attn"] + call_ms["lm"]
    pair_gbs = (ab["attn"] + ab["lm"]) / (pair_ms * 1e-3) / 1e9

    result = {
        "metric": "decode tokens/s at fixed concurrency C; achieved HBM GB/s vs MI355X peak",
        "value": round(cfg.C / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": max(0, SETTLE_STEPS - args.warmup),
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == W.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): C={cfg.C}, {cfg.Hq}q/{cfg.Hkv}kv heads, "
                               f"head_dim {cfg.D}, page {cfg.page_size}, mean ctx {inp['ctx_len'].mean():.0f}, "
                               f"LM head {cfg.H}x{cfg.V}; + IS batch of {isb['B']} trajectories, {isb['N']} tokens "
                               f"(rotating over {len(isd)} copies)",
                   "step": "decode_attn (1 layer) + lmhead_logprob + is_ratio", "concurrency": cfg.C},
        "roofline": roofline,
        "call_ms": call,
        "attn_plus_lm": {"algorithmic_GB": round((ab["attn"] + ab["lm"]) / 1e9, 4), "median_ms": round(pair_ms, 4),
                         "achieved_GBps": round(pair_gbs, 1), "frac_hbm": round(pair_gbs / HBM_PEAK_GBS, 4),
                         "decode_tokens_per_s_attn_lm_only": round(cfg.C / (pair_ms * 1e-3), 1),
                         "projection_28_layers": {
                             "tokens_per_s": round(cfg.C / ((28 * call_ms["attn"] + call_ms["lm"]) * 1e-3), 1),
                             "note": "context only: C / (28 x attention call + LM-head call), 28 = the layer count of "
                                     "a 7B decoder of this shape; the other work of a layer is not part of the path"}},
        "kernels": kernels,
        "all_kernel_ms": {k: round(v, 4) for k, v in kernel_ms.items()},
        "input_generation_s": round(t_gen, 1),
    }

    # ---- the practical ceilings the fractions lean on, measured in this run ----
    limits = {"device_copy_1GiB_GBps": round(device_copy_1gib(), 1)}
    limits["device_copy_frac_hbm"] = round(limits["device_copy_1GiB_GBps"] / HBM_PEAK_GBS, 4)
    if cfg.dtype == W.BF16 and not args.no_extras:
        sampler = ClockSampler()
        mhz_n, ms_n = sampler.measure(lambda: lm.run(stream), 1.0)
        pw_n = sampler.last_power_w
        zero = clone_device(lm)
        zero.hidden.zero_()
        zero.weight.zero_()
        mhz_z, ms_z = sampler.measure(lambda: zero.run(stream), 1.0)
        pw_z = sampler.last_power_w
        del zero
        limits["lmhead_core_clock"] = {
            "seeded_operands": {"sclk_MHz": mhz_n, "ms_per_call": ms_n, "board_power_W": pw_n},
            "zero_operands": {"sclk_MHz": mhz_z, "ms_per_call": ms_z, "board_power_W": pw_z},
            "how": "medians of the driver's current sclk level and of hwmon power1_input, sampled every 5 ms over "
                   "1 s of back-to-back calls"}
        mhz_a, ms_a = sampler.measure(lambda: attn.run(stream), 1.0)
        limits["decode_attn_core_clock"] = {"sclk_MHz": mhz_a, "ms_per_call": ms_a,
                                            "board_power_W": sampler.last_power_w}
        limits["board_power_cap_W"] = sampler.power_cap_w()
    result["limits"] = limits
    extras = result["extras"] = {}

    if not args.no_extras:
        # ---- the GRPO clipped surrogate on the same IS batch (same 17 algorithmic bytes per
        # token as the ratio kernel), rotating over distinct copies ----
        gd = [runner.stage_grpo_surrogate(isb, dev) for _ in range(CACHE_ROTATION_SETS)]
        g_ms = time_rotating([(lambda d=d: d.run(stream)) for d in gd], stream, args.steps, 8)
        gm = float(np.median(g_ms))
        extras["grpo_surrogate"] = {"call_ms": dist(g_ms), "algorithmic_bytes": ab["is"],
                                    "achieved_GBps": round(ab["is"] / (gm * 1e-3) / 1e9, 1),
                                    "workload": f"IS batch of {isb['B']} trajectories, {isb['N']} tokens, "
                                                f"rotating over {len(gd)} copies"}
        del gd
        i_ms = time_rotating([(lambda d=d: d.run(stream)) for d in isd], stream, args.steps, 8)
        extras["is_ratio"] = {"call_ms": dist(i_ms), "algorithmic_bytes": ab["is"],
                              "achieved_GBps": round(ab["is"] / (float(np.median(i_ms)) * 1e-3) / 1e9, 1),
                              "workload": f"the step's IS batch on its own, rotating over {len(isd)} copies"}
    # ---- the same step captured in a HIP graph: eight consecutive steps (one per copy of the
    # IS batch, so the rotation is kept) recorded once and replayed; the library enqueues
    # kernels only, so nothing else has to change for a caller that replays its decode loop ----
    if args.config == 2 and not args.no_extras:
        gs = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gs):
            cs = torch.cuda.current_stream()
            for k in range(len(isd)):
                attn.run(cs)
                lm.run(cs)
                isd[k].run(cs)
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        n_rep = max(args.steps // len(isd), 4)
        gev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_rep)]
        for e0, e1 in gev:
            e0.record(stream)
            graph.replay()
            e1.record(stream)
        torch.cuda.synchronize()
        g_ms = [e0.elapsed_time(e1) / len(isd) for e0, e1 in gev]
        extras["graph_step"] = {"ms_per_step": dist(g_ms), "steps_per_graph": len(isd), "replays": n_rep,
                                "tokens_per_s": round(cfg.C / (float(np.median(g_ms)) * 1e-3), 1),
                                "workload": "the timed step, eight of them captured in one HIP graph and replayed"}
        del graph

    # ---- the 1.5B-shaped step (config 1): attention + LM head, reported without a bar.  Its KV
    # (129 MB) fits the Infinity Cache, so the calls rotate over distinct copies ----
    if args.config == 2 and not args.no_extras:
        cfg1 = W.DECODE_CONFIGS[1]
        inp1 = W.make_decode_inputs(cfg1)
        ab1 = algorithmic_bytes(cfg1, inp1, None)
        a1 = [runner.stage_attn(inp1, cfg1.dtype, dev)]
        l1 = [runner.stage_lmhead(inp1, cfg1.dtype, dev)]
        for _ in range(3):
            a1.append(clone_device(a1[0]))
            l1.append(clone_device(l1[0]))
        a_ms = time_rotating([(lambda d=d: d.run(stream)) for d in a1], stream, args.steps, 12)
        l_ms = time_rotating([(lambda d=d: d.run(stream)) for d in l1], stream, args.steps, 12)
        am, lmm = float(np.median(a_ms)), float(np.median(l_ms))
        extras["config1_step"] = {
            "attn_call_ms": dist(a_ms), "lm_call_ms": dist(l_ms),
            "attn_GBps": round(ab1["attn"] / (am * 1e-3) / 1e9, 1), "lm_GBps": round(ab1["lm"] / (lmm * 1e-3) / 1e9, 1),
            "attn_frac_hbm": round(ab1["attn"] / (am * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "lm_frac_hbm": round(ab1["lm"] / (lmm * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "decode_tokens_per_s_attn_lm_only": round(cfg1.C / ((am + lmm) * 1e-3), 1),
            "workload": f"config 1 ({cfg1.name}): C={cfg1.C}, {cfg1.Hq}q/{cfg1.Hkv}kv heads, mean ctx "
                        f"{inp1['ctx_len'].mean():.0f}, LM head {cfg1.H}x{cfg1.V}; rotating over {len(a1)} copies"}
        del a1, l1, inp1
    # ---- log-probs of given tokens under the current policy for one micro-batch of M
    # positions (the recomputed side of the ratio), a dense contraction ----
    if cfg.H > 0 and args.config == 2 and not args.no_extras:
        M = args.token_logprob_m
        tb = W.make_token_logprob_inputs(cfg, M)
        td = runner.stage_token_logprob(tb["hidden"], None, tb["tokens"], tb["temperature"], cfg.dtype, dev,
                                        weight_dev=lm.weight)
        t_ms = time_rotating([lambda: td.run(stream)], stream, max(5, args.steps // 5), 3)
        tl_ms = float(np.median(t_ms))
        flops = 2.0 * M * cfg.H * cfg.V
        extras["token_logprob"] = {
            "call_ms": dist(t_ms), "M": M, "positions_per_s": round(M / (tl_ms * 1e-3), 1),
            "TFLOPs": round(flops / (tl_ms * 1e-3) / 1e12, 1),
            "mfma_frac": round(flops / (tl_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": traffic.get("lmhead_gemm_given_kernel"),
            "workload": f"{M} positions x LM head {cfg.H}x{cfg.V} bf16, given tokens"}
        cs = ClockSampler()
        mhz, _ms = cs.measure(lambda: td.run(stream), 1.0)
        extras["token_logprob"].update({"sclk_MHz": mhz, "board_power_W": cs.last_power_w})
        del td
    # ---- re-prefill attention of resumed partial trajectories (one layer): a handful of
    # buffered trajectories with the config's length recipe ----
    if args.config == 2 and not args.no_extras:
        plens = W.make_ctx_len(cfg, np.random.default_rng(cfg.seed + 5))[:args.prefill_seqs]
        pb = W.make_prefill_case(cfg.seed + 6, plens, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype)
        pd = runner.stage_prefill_attn(pb, cfg.dtype, dev)
        p_ms = time_rotating([lambda: pd.run(stream)], stream, max(5, args.steps // 5), 3)
        pf_ms = float(np.median(p_ms))
        L = plens.astype(np.float64)
        pflops = float((4.0 * cfg.Hq * cfg.D * L * (L + 1) / 2).sum())
        extras["prefill_attn"] = {
            "call_ms": dist(p_ms), "tokens": int(plens.sum()),
            "tokens_per_s": round(float(plens.sum()) / (pf_ms * 1e-3), 1),
            "TFLOPs": round(pflops / (pf_ms * 1e-3) / 1e12, 1),
            "mfma_frac": round(pflops / (pf_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": traffic.get("prefill_attn_kernel"),
            "workload": f"{len(plens)} resumed trajectories, lengths {int(plens.min())}..{int(plens.max())}, "
                        f"{cfg.Hq}q/{cfg.Hkv}kv heads, causal, one layer"}
        cs = ClockSampler()
        mhz, _ms = cs.measure(lambda: pd.run(stream), 1.0)
        extras["prefill_attn"].update({"sclk_MHz": mhz, "board_power_W": cs.last_power_w})
        del pd, pb
    # ---- decode attention on the long-tail stress configuration (resumed 32k-token
    # trajectories among short ones: what the split along the context is for) ----
    if args.config == 2 and not args.no_longtail and not args.no_extras:
        cfg3 = W.DECODE_CONFIGS[3]
        inp3 = W.make_decode_inputs(cfg3, with_lmhead=False)
        a3 = runner.stage_attn(inp3, cfg3.dtype, dev)
        lt = time_rotating([lambda: a3.run(stream)], stream, args.steps, 10)
        lt_ms = float(np.median(lt))
        ctx3 = inp3["ctx_len"].astype(np.int64)
        kv3 = int(ctx3.sum()) * 2 * cfg3.Hkv * cfg3.D * cfg3.elem_bytes
        extras["decode_attn_longtail"] = {
            "call_ms": dist(lt), "kv_bytes": kv3, "achieved_GBps": round(kv3 / (lt_ms * 1e-3) / 1e9, 1),
            "frac_hbm": round(kv3 / (lt_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "workload": f"config 3 ({cfg3.name}): C={cfg3.C}, ctx {int(ctx3.min())}..{int(ctx3.max())}, "
                        f"{int((ctx3 == ctx3.max()).sum())} sequences at the maximum"}
        del a3, inp3
    # ---- host only: the rollout manager's schedule for 20 training steps at the paper's
    # settings (Table 4: 64 inputs x 8 samples per step, pool 1024) ----
    if args.config == 2 and not args.no_extras:
        rngs = np.random.default_rng(cfg.seed + 9)
        n_in, n_s, n_b, n_pool, n_st = 64 * 40, 8, 64, 1024, 20
        rl = np.minimum(np.maximum(np.rint(rngs.lognormal(7.5, 1.1, size=(n_in, n_s))), 1), 16384).astype(np.int32)
        pl = np.full(n_in, cfg.prompt, dtype=np.int32)
        t0s = time.perf_counter()
        sched = binding.rollout_schedule(pl, rl, n_pool, n_b, max_stages=n_st)
        t_sched = time.perf_counter() - t0s
        bt = sum(x["batch_tokens"] for x in sched)
        extras["rollout_schedule"] = {
            "host_ms": round(t_sched * 1e3, 2), "stages": len(sched), "pool": n_pool,
            "decode_steps": sum(x["steps"] for x in sched),
            "offpolicy_token_frac": round(sum(x["batch_offpolicy"] for x in sched) / max(bt, 1), 4),
            "reprefill_tokens_per_generated": round(sum(x["reprefill_tokens"] for x in sched)
                                                    / max(sum(x["generated"] for x in sched), 1), 4),
            "pool_idle_frac": round(sum(x["slot_steps_idle"] for x in sched)
                                    / max(n_pool * sum(x["steps"] for x in sched), 1), 4),
            "workload": f"{n_st} training steps of {n_b} inputs x {n_s} samples, response lengths of the config-2 recipe"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, inp, args.cpu_sample)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
