#!/usr/bin/env python3
"""Benchmark of the CoPRIS rollout-decode hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic input:
  copris_decode_attn (work list, split-K attention, merge: one layer's KV) +
  copris_lmhead_logprob (LM head + log-softmax + Gumbel-max + log-prob gather)
on the 7B-shaped C=256 decode configuration, + copris_is_ratio on the cross-stage IS
batch (256 trajectories).  All inputs are resident in HBM before the timed region.

Prints ONE JSON line: decode tokens/s (C / step time), the HBM roofline of the dominant
kernel (algorithmic bytes / kernel duration measured with events around that kernel's
launches, vs 8 TB/s) and the fp64 CPU oracle timed on a bounded sample of the same
workload on this machine's host cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, choices=[0, 1, 2],
                    help="decode config index (2 = the 7B-shaped C=256 config the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=256, help="sequences in the oracle sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic: the scale for the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    ap.add_argument("--token-logprob-m", type=int, default=8192,
                    help="positions in the micro-batch of the given-token log-prob measurement")
    ap.add_argument("--no-longtail", action="store_true",
                    help="skip the decode-attention measurement on the long-tail stress configuration")
    ap.add_argument("--prefill-seqs", type=int, default=16,
                    help="resumed trajectories in the re-prefill attention measurement")
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
    is_ = 17 * int(isb["N"])                                    # cur + selected old + mask in, 2 outputs
    return {"attn": attn, "lm": lm, "is": is_, "kv": kv}


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


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_05589_amd import binding, runner, workloads as W

    dev = runner.require_gpu()
    cfg = W.DECODE_CONFIGS[args.config]
    t_gen = time.perf_counter()
    inp = W.make_decode_inputs(cfg)
    isb = W.make_is_inputs(W.IS_CONFIGS[4 if args.config != 0 else 0])
    t_gen = time.perf_counter() - t_gen

    attn = runner.stage_attn(inp, cfg.dtype, dev)
    lm = runner.stage_lmhead(inp, cfg.dtype, dev)
    isd = runner.stage_is_ratio(isb, dev)
    stream = torch.cuda.current_stream()
    ab = algorithmic_bytes(cfg, inp, isb)

    def step():
        attn.run(stream)
        lm.run(stream)
        isd.run(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

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
        isd.run(stream)
        ev[k][3].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    call_ms = {name: float(np.mean([ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(args.steps)]))
               for i, name in enumerate(["attn", "lm", "is"])}

    # ---- per-kernel durations: the library's launch hook records an event before and
    # after every kernel launch (same stream, same K steps, instrumented pass) ----
    recs = []

    def hook(kernel, phase, _stream, _user):
        e = torch.cuda.Event(enable_timing=True)
        e.record(stream)
        recs.append((kernel.decode(), phase, e))

    binding.set_launch_hook(hook)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    binding.set_launch_hook(None)
    kernel_ms = {}
    for i in range(0, len(recs), 2):
        (name, p0, e0), (name1, p1, e1) = recs[i], recs[i + 1]
        assert name == name1 and p0 == 0 and p1 == 1
        kernel_ms.setdefault(name, []).append(e0.elapsed_time(e1))
    kernel_ms = {k: float(np.mean(v)) for k, v in kernel_ms.items()}

    # ---- roofline of the dominant kernel ----
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
        kernels[kname] = {"avg_ms": round(kernel_ms[kname], 4), "algorithmic_bytes": ab[part],
                          "achieved_GBps": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4),
                          "traffic": traffic.get(kname)}
    lm_flops = 2.0 * cfg.C * cfg.H * cfg.V
    kernels[main_kernels["lm"]]["mfma_frac"] = round(
        lm_flops / (kernel_ms[main_kernels["lm"]] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)
    dom = max((main_kernels["attn"], main_kernels["lm"]), key=lambda k: kernel_ms[k])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kernels[dom]["achieved_GBps"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": kernels[dom]["frac_hbm"],
                "traffic": kernels[dom]["traffic"], "avg_kernel_ms": kernels[dom]["avg_ms"]}
    pair_gbs = (ab["attn"] + ab["lm"]) / ((call_ms["attn"] + call_ms["lm"]) * 1e-3) / 1e9

    result = {
        "metric": "decode tokens/s at fixed concurrency C; achieved HBM GB/s vs MI355X peak",
        "value": round(cfg.C / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg.dtype == W.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index} ({cfg.name}): C={cfg.C}, {cfg.Hq}q/{cfg.Hkv}kv heads, "
                               f"head_dim {cfg.D}, page {cfg.page_size}, mean ctx {inp['ctx_len'].mean():.0f}, "
                               f"LM head {cfg.H}x{cfg.V}; + IS batch of {isb['B']} trajectories, {isb['N']} tokens",
                   "step": "decode_attn (1 layer) + lmhead_logprob + is_ratio", "concurrency": cfg.C},
        "roofline": roofline,
        "call_ms": {k: round(v, 4) for k, v in call_ms.items()},
        "attn_plus_lm": {"algorithmic_GB": round((ab["attn"] + ab["lm"]) / 1e9, 4),
                         "achieved_GBps": round(pair_gbs, 1), "frac_hbm": round(pair_gbs / HBM_PEAK_GBS, 4),
                         "decode_tokens_per_s_attn_lm_only": round(cfg.C / ((call_ms["attn"] + call_ms["lm"]) * 1e-3), 1)},
        "kernels": kernels,
        "all_kernel_ms": {k: round(v, 4) for k, v in kernel_ms.items()},
        "input_generation_s": round(t_gen, 1),
    }
    # ---- outside the step: the GRPO clipped surrogate on the same IS batch (a row added
    # after the decode path; same 17 algorithmic bytes per token as the ratio kernel) ----
    gd = runner.stage_grpo_surrogate(isb, dev)
    for _ in range(3):
        gd.run(stream)
    torch.cuda.synchronize()
    g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    g0.record(stream)
    for _ in range(args.steps):
        gd.run(stream)
    g1.record(stream)
    torch.cuda.synchronize()
    grpo_ms = g0.elapsed_time(g1) / args.steps
    result["extras"] = {"grpo_surrogate": {"call_ms": round(grpo_ms, 4), "algorithmic_bytes": ab["is"],
                                           "achieved_GBps": round(ab["is"] / (grpo_ms * 1e-3) / 1e9, 1),
                                           "workload": f"IS batch of {isb['B']} trajectories, {isb['N']} tokens"}}
    # ---- outside the step: log-probs of given tokens under the current policy for one
    # micro-batch of M positions (the recomputed side of the ratio), a dense contraction ----
    if cfg.H > 0 and args.config == 2:
        M = args.token_logprob_m
        tb = W.make_token_logprob_inputs(cfg, M)
        td = runner.stage_token_logprob(tb["hidden"], None, tb["tokens"], tb["temperature"], cfg.dtype, dev,
                                        weight_dev=lm.weight)
        for _ in range(2):
            td.run(stream)
        torch.cuda.synchronize()
        reps = max(3, args.steps // 5)
        t0e, t1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0e.record(stream)
        for _ in range(reps):
            td.run(stream)
        t1e.record(stream)
        torch.cuda.synchronize()
        tl_ms = t0e.elapsed_time(t1e) / reps
        flops = 2.0 * M * cfg.H * cfg.V
        result["extras"]["token_logprob"] = {
            "call_ms": round(tl_ms, 3), "M": M, "positions_per_s": round(M / (tl_ms * 1e-3), 1),
            "TFLOPs": round(flops / (tl_ms * 1e-3) / 1e12, 1),
            "mfma_frac": round(flops / (tl_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "workload": f"{M} positions x LM head {cfg.H}x{cfg.V} bf16, given tokens"}
    # ---- outside the step: re-prefill attention of resumed partial trajectories (one
    # layer): a handful of buffered trajectories with the config's length recipe ----
    if args.config == 2:
        plens = W.make_ctx_len(cfg, np.random.default_rng(cfg.seed + 5))[:args.prefill_seqs]
        pb = W.make_prefill_case(cfg.seed + 6, plens, cfg.Hq, cfg.Hkv, cfg.D, cfg.dtype)
        pd = runner.stage_prefill_attn(pb, cfg.dtype, dev)
        for _ in range(2):
            pd.run(stream)
        torch.cuda.synchronize()
        reps = max(3, args.steps // 5)
        p0e, p1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0e.record(stream)
        for _ in range(reps):
            pd.run(stream)
        p1e.record(stream)
        torch.cuda.synchronize()
        pf_ms = p0e.elapsed_time(p1e) / reps
        L = plens.astype(np.float64)
        pflops = float((4.0 * cfg.Hq * cfg.D * L * (L + 1) / 2).sum())
        result["extras"]["prefill_attn"] = {
            "call_ms": round(pf_ms, 3), "tokens": int(plens.sum()),
            "tokens_per_s": round(float(plens.sum()) / (pf_ms * 1e-3), 1),
            "TFLOPs": round(pflops / (pf_ms * 1e-3) / 1e12, 1),
            "mfma_frac": round(pflops / (pf_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "workload": f"{len(plens)} resumed trajectories, lengths {int(plens.min())}..{int(plens.max())}, "
                        f"{cfg.Hq}q/{cfg.Hkv}kv heads, causal, one layer"}
        del pd, pb
    # ---- outside the step: decode attention on the long-tail stress configuration (resumed
    # 32k-token trajectories among short ones: what the split along the context is for) ----
    if args.config == 2 and not args.no_longtail:
        cfg3 = W.DECODE_CONFIGS[3]
        inp3 = W.make_decode_inputs(cfg3, with_lmhead=False)
        a3 = runner.stage_attn(inp3, cfg3.dtype, dev)
        for _ in range(5):
            a3.run(stream)
        torch.cuda.synchronize()
        l0e, l1e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        l0e.record(stream)
        for _ in range(args.steps):
            a3.run(stream)
        l1e.record(stream)
        torch.cuda.synchronize()
        lt_ms = l0e.elapsed_time(l1e) / args.steps
        ctx3 = inp3["ctx_len"].astype(np.int64)
        kv3 = int(ctx3.sum()) * 2 * cfg3.Hkv * cfg3.D * cfg3.elem_bytes
        result["extras"]["decode_attn_longtail"] = {
            "call_ms": round(lt_ms, 4), "kv_bytes": kv3, "achieved_GBps": round(kv3 / (lt_ms * 1e-3) / 1e9, 1),
            "frac_hbm": round(kv3 / (lt_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "workload": f"config 3 ({cfg3.name}): C={cfg3.C}, ctx {int(ctx3.min())}..{int(ctx3.max())}, "
                        f"{int((ctx3 == ctx3.max()).sum())} sequences at the maximum"}
        del a3, inp3
    # ---- outside the step, host only: the rollout manager's schedule for 20 training steps
    # at the paper's settings (Table 4: 64 inputs x 8 samples per step, pool 1024) ----
    if args.config == 2:
        rngs = np.random.default_rng(cfg.seed + 9)
        n_in, n_s, n_b, n_pool, n_st = 64 * 40, 8, 64, 1024, 20
        rl = np.minimum(np.maximum(np.rint(rngs.lognormal(7.5, 1.1, size=(n_in, n_s))), 1), 16384).astype(np.int32)
        pl = np.full(n_in, cfg.prompt, dtype=np.int32)
        t0s = time.perf_counter()
        sched = binding.rollout_schedule(pl, rl, n_pool, n_b, max_stages=n_st)
        t_sched = time.perf_counter() - t0s
        bt = sum(x["batch_tokens"] for x in sched)
        result["extras"]["rollout_schedule"] = {
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
