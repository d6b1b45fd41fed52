#!/usr/bin/env python3
"""Decode-throughput benchmark of the DMTD hot path on one MI355X.

Workload: the Qwen3-4B-shaped batch-1 configuration (36 layers, 1024-token prompt, 512
generated tokens, tau=3, n_late=8) with seeded synthetic weights and prompt.  A "step" is
one decode cycle (one full pass + tau-1 late-only passes = tau tokens).  Cycles are enqueued
several at a time (dmtd_decode; --cycles-per-call, default 8: the host collects the tokens
after every 8 cycles) and the rate with one blocking call per cycle is reported beside it.
The same run also times tau=1 (ordinary decoding) on the same kernels, the host collecting
after as many tokens, the dominant kernel on its own with HIP events (roofline), and the CPU
oracle on a bounded sample (cpu_baseline).
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def algorithmic_bytes(sh, n_late, ctx_full, ctx_late_list, batch, n_early=0):
    """Bytes one decode cycle must move (each needed weight byte once per step, each live KV byte of a
    visited layer once per step); returns (cycle bytes, per-layer weight bytes, table bytes)."""
    e = sh.elem_bytes
    d, hd = sh.hidden, sh.head_dim
    per_layer = e * (2 * d + 2 * hd + d * (sh.n_q_heads + 2 * sh.n_kv_heads) * hd + d * sh.n_q_heads * hd
                     + 3 * d * sh.intermediate)
    table = e * (sh.vocab * d + d)
    kv_tok = 2 * sh.n_kv_heads * hd * e * batch      # per layer per cached position
    total = sh.n_layers * per_layer + table + sh.n_layers * kv_tok * ctx_full
    for c in ctx_late_list:
        total += (n_early + n_late) * per_layer + table + (n_early + n_late) * kv_tok * c
    return total, per_layer, table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=160, help="timed decode cycles (tau tokens each)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--tau", type=int, default=0, help="override the workload's cycle length")
    ap.add_argument("--n-late", type=int, default=0, help="override the workload's number of decoding layers")
    ap.add_argument("--n-early", type=int, default=0, help="ExDy variant: encoding layers the in-cycle tokens reuse (0 = plain method)")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--cycles-per-call", type=int, default=8,
                    help="cycles enqueued per dmtd_decode call, i.e. how often the host collects the tokens (the tau=1 leg "
                         "collects after the same number of tokens); 0: one dmtd_decode_cycle call per cycle")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graphs", action="store_true")
    ap.add_argument("--counters-run", action="store_true",
                    help="short run for rocprofv3 --pmc: 64-token prompt, DMTD leg only, no kernel timing (counter "
                         "collection serialises every dispatch); prints no benchmark line")
    ap.add_argument("--table3", action="store_true",
                    help="the paper's speed-test grid instead of the benchmark line: batch 1, 2, 4, 8 x tau 1..4 at a 1024-token "
                         "prompt, 1024 generated tokens per sequence, whole generation timed (decode steps only); prints one JSON line")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 1 GiB device copies first (known traffic, to scale rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import dmtd_inputs as di
    import paper_2510_11958_amd as pkg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the decode path has no CPU fallback", file=sys.stderr)
        sys.exit(1)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB per launch
        torch.cuda.synchronize()
        del src, dst

    wl = di.WORKLOADS[args.workload]
    if args.table3:
        table3(args, di, pkg, torch, np, wl)
        return
    sh, B, P, tau, n_late = wl.shape, wl.batch, wl.prompt_len, wl.tau, wl.n_late
    tau, n_late, B = args.tau or tau, args.n_late or n_late, args.batch or B
    n_early = args.n_early
    if args.counters_run:
        P = 64
    K, W = args.steps, args.warmup
    t0 = time.time()
    blob = di.make_weight_blob(sh, seed=0)
    prompts = di.make_prompts(sh.vocab, B, P, seed=1)
    max_seq = P + 1 + (K + W + 2) * max(tau, 1) + 8
    cfg = pkg.ModelConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab,
                          dtype=sh.dtype, max_batch=B, max_seq_len=max_seq, use_graphs=not args.no_graphs)
    eng = pkg.Engine(cfg, blob)
    if n_early:
        eng.set_n_early(n_early)
    t_setup = time.time() - t0

    prefill_ms = []

    def run(tau_run, cycles, warm, per_call):
        """Times exactly `cycles` cycles of tau_run tokens.  per_call > 0: dmtd_decode calls of up to per_call cycles, enqueued
        as one piece of GPU work each, the host collecting the tokens at the end of a call; 0: one blocking
        dmtd_decode_cycle call per cycle."""
        eng.reset()
        torch.cuda.synchronize()
        tp = time.perf_counter()
        eng.prefill(prompts)                              # synchronises before it returns the first tokens
        prefill_ms.append((time.perf_counter() - tp) * 1e3)
        eng.decode_cycle(tau_run, n_late)                 # finishes cycle 1 (tau-1 tokens); untimed
        for _ in range(warm):
            eng.decode_cycle(tau_run, n_late)
        if per_call:
            eng.decode(tau_run, n_late, tau_run)          # one untimed cycle through the entry point being timed
        torch.cuda.synchronize()
        ctx0 = eng.state()["n_tok"]
        t = time.perf_counter()
        ntok, left = 0, cycles
        while left > 0:
            if per_call:
                c = min(left, per_call, 64 // tau_run)
                ntok += eng.decode(tau_run, n_late, c * tau_run).shape[1] * B
            else:
                c = 1
                ntok += eng.decode_cycle(tau_run, n_late).shape[1] * B
            left -= c
        torch.cuda.synchronize()
        dt = time.perf_counter() - t
        assert ntok == cycles * tau_run * B
        return ntok, dt, ctx0

    cpc = max(0, min(args.cycles_per_call, 64 // tau))
    ntok, dt, ctx0 = run(tau, K, W, cpc)
    if args.counters_run:
        print(f"counters run done: {ntok} tokens", file=sys.stderr)
        return
    # tau = 1 on the same kernels, over the same number of tokens
    ntok1, dt1, _ = run(1, K * tau, W * tau, cpc * tau)
    # the same cycles with one blocking call per cycle (the host between all cycles), for reference
    ntok_pc, dt_pc, _ = run(tau, K, W, 0) if cpc else (ntok, dt, ctx0)

    # algorithmic bytes of the timed DMTD cycles (true per-step context)
    total_bytes = 0
    for c in range(K):
        base = ctx0 + c * tau
        cyc, per_layer, table = algorithmic_bytes(sh, n_late, base + 1, [base + 1 + i for i in range(1, tau)], B, n_early)
        total_bytes += cyc
    e2e_gbs = total_bytes / dt / 1e9

    # roofline of the dominant kernel: RMSNorm + gate/up + SwiGLU weight stream (49 % of a layer's bytes),
    # launched once per layer back to back, HIP-event timed on the engine's stream, with the activation rows of
    # this workload's full step (batch x rows per sequence) and of its late-only step (batch)
    rows = min(B * min(tau, 4), B * 16)
    rows_late = B
    reps = 10
    per = {}
    r_seq = min(tau, 4)
    for kind, r in (("gateup", rows), ("gateup", rows_late), ("down", rows), ("down", rows_late), ("qkv", rows), ("qkv", rows_late),
                    ("oproj", rows), ("oproj", rows_late), ("lmhead", B), ("attn", 1), ("attn", r_seq)):
        per[f"{kind}_m{r}"] = eng.time_kernel(kind, r, reps)
    # what a launch that only reads the same weight bytes takes (no activations, no arithmetic, no output)
    read_only = {}
    if sh.elem_bytes == 2:
        read_only = {k: eng.time_kernel("read_" + k, 1, reps) for k in ("gateup", "down", "qkv", "oproj")}
    # the same kernel times summed over one cycle's launches (full step: front layers with the refill rows, late layers
    # and LM head with one row per sequence; tau-1 late-only steps), to set beside ms_per_step
    layer_full = sum(per[f"{k}_m{rows}"] for k in ("qkv", "oproj", "gateup", "down")) + per[f"attn_m{r_seq}"]
    layer_late = sum(per[f"{k}_m{rows_late}"] for k in ("qkv", "oproj", "gateup", "down")) + per["attn_m1"]
    n_front = sh.n_layers - n_late - n_early
    kernel_us_cycle = (n_front * layer_full + (n_late + n_early) * layer_late + per[f"lmhead_m{B}"]
                       + (tau - 1) * ((n_late + n_early) * layer_late + per[f"lmhead_m{B}"]))
    gu_bytes = 2 * sh.intermediate * sh.hidden * sh.elem_bytes + sh.hidden * sh.elem_bytes
    achieved = gu_bytes / (per[f"gateup_m{rows}"] * 1e-6) / 1e9
    traffic, traffic_source = measured_traffic(args.workload)
    kernel_name = "gemv_mfma_kernel<SWIGLU, NORM>" if rows <= 5 else "gemm_mfma_kernel<SWIGLU, NORM> (+ gemm_finish_kernel)"
    roofline = {"bound": "hbm", "kernel": f"{kernel_name} with {rows} rows (RMSNorm + gate/up + SwiGLU)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "bytes_per_launch": gu_bytes, "avg_launch_us": round(per[f"gateup_m{rows}"], 2),
                "other_kernels_us": {k: round(v, 2) for k, v in per.items()}}
    if read_only:
        roofline["read_only_kernel_us"] = {k: round(v, 2) for k, v in read_only.items()}
        roofline["frac_of_read_only_kernel"] = round(read_only["gateup"] / per[f"gateup_m{rows}"], 4)
    if rows > 16:
        # batched steps run on the matrix cores in earnest: flops of the same launch (two bf16 activation planes, so
        # 2 x 2 x rows x N x K multiply-adds) against the dense bf16 peak; the launch stays bound by the weight stream
        flops = 2.0 * 2.0 * rows * (2 * sh.intermediate) * sh.hidden
        tf = flops / (per[f"gateup_m{rows}"] * 1e-6) / 1e12
        roofline["mfma"] = {"flops_per_launch": flops, "achieved_TFLOPs": round(tf, 1), "peak_TFLOPs": MFMA_BF16_PEAK_TFLOPS,
                            "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(di, blob, sh, tau, n_late, P)

    out = {
        "metric": "decode tokens/sec at 1 GPU (DMTD tau vs tau=1) + achieved HBM GB/s fraction",
        "value": round(ntok / dt, 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(dt / K * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if sh.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name + ("" if (tau, n_late, B, n_early) == (wl.tau, wl.n_late, wl.batch, 0) else
                                          f" [run with tau={tau}, n_late={n_late}, n_early={n_early}, batch={B}]"), "tau": tau, "n_late": n_late, "n_early": n_early, "batch": B, "prompt_len": P,
                   "context_at_start": ctx0, "graphs": not args.no_graphs, "cycles_per_call": cpc},
        "one_call_per_cycle_tokens_per_s": round(ntok_pc / dt_pc, 2),
        "tau1_tokens_per_s": round(ntok1 / dt1, 2), "speedup_vs_tau1": round((ntok / dt) / (ntok1 / dt1), 4),
        "end_to_end": {"algorithmic_GB_per_cycle": round(total_bytes / K / 1e9, 4), "achieved_GBs": round(e2e_gbs, 1),
                       "frac_of_hbm_peak": round(e2e_gbs / HBM_PEAK_GBS, 4)},
        "kernel_us_sum_per_cycle": round(kernel_us_cycle, 1),
        "prefill_ms": round(min(prefill_ms), 2),          # untimed by the metric: the whole prompt batch through all layers, host call to first tokens
        "roofline": roofline, "cpu_baseline": cpu, "setup_s": round(t_setup, 1),
    }
    print(json.dumps(out))


def table3(args, di, pkg, torch, np, wl):
    """The grid of the paper's speed test (Sec. 3.4, Table 3): 1024 random prompt tokens, 1024 generated tokens per
    sequence, batch 1 / 2 / 4 / 8, ordinary decoding (tau = 1) and cycle lengths 2, 3, 4 with the last n_late layers
    reused.  Timed: everything after prefill (the first token comes from prefill), i.e. 1023 decode steps' tokens per
    sequence, through dmtd_decode calls of up to 64 steps; tokens/s = batch * 1023 / time."""
    sh, n_late = wl.shape, args.n_late or wl.n_late
    P, G = 1024, 1024
    blob = di.make_weight_blob(sh, seed=0)
    dev = torch.from_numpy(blob.view(np.int16)).cuda()
    grid = {}
    for B in (1, 2, 4, 8):
        cfg = pkg.ModelConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab,
                              dtype=sh.dtype, max_batch=B, max_seq_len=P + G + 8, use_graphs=not args.no_graphs)
        eng = pkg.Engine(cfg, dev)
        prompts = di.make_prompts(sh.vocab, B, P, seed=1)
        for tau in (1, 2, 3, 4):
            best = None
            for rep in range(2):                      # the first pass also captures the graphs of every context bucket
                eng.reset()
                eng.prefill(prompts)
                torch.cuda.synchronize()
                t = time.perf_counter()
                left = G - 1
                while left > 0:
                    n = min(left, 64 // tau * tau if left >= tau else left)
                    left -= eng.decode(tau, n_late, n).shape[1]
                torch.cuda.synchronize()
                dt = time.perf_counter() - t
                best = dt if best is None else min(best, dt)
            assert eng.state()["n_tok"] == P + G - 1
            grid[f"B{B}_tau{tau}"] = round(B * (G - 1) / best, 1)
        eng.close()
    out = {"table3": grid, "unit": "tokens/s", "prompt_len": P, "generated": G, "n_late": n_late,
           "speedup_vs_tau1": {k: round(v / grid[k.split("_")[0] + "_tau1"], 3) for k, v in grid.items()},
           "paper_speedup_batch1_a100": {"tau2": 1.44, "tau3": 1.85, "tau4": 2.15},
           "workload": f"{wl.shape.n_layers}-layer 4B shape, P={P}, G={G}, n_late={n_late}, graphs {not args.no_graphs}"}
    print(json.dumps(out))


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE +
    WRITE_SIZE, scaled by what the same counters read for a plain copy of known size), and where that figure comes
    from: counters cannot be collected inside this run (collection serialises every dispatch), so the figure is the
    one of the last counter run of this kernel, named with its commit and date.  (None, None) if there is none."""
    rel = os.path.join("profiles", f"gateup_swiglu_{workload}_pmc.txt")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            d = json.load(f)
        run = d.get("counter_run", {})
        return d["traffic_bytes_per_launch"], {"file": rel, "commit": run.get("commit"), "date": run.get("date"),
                                               "measured_in_this_run": False}
    except Exception:
        return None, None


def cpu_baseline(di, blob, sh, tau, n_late, prompt_len):
    """The NumPy oracle, as it stands, on this machine's host cores: decode tokens/s on a bounded sample."""
    import numpy as np
    from oracle import dmtd_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    ocfg = O.OracleConfig(sh.n_layers, sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.intermediate, sh.vocab,
                          sh.rms_eps, sh.rope_theta, sh.tied_embeddings)
    big = di.blob_elems(sh) > 1_000_000_000
    dt = np.float32 if big else np.float64
    w = O.unpack_weights(blob, ocfg, dt)
    P = min(prompt_len, 1024)      # the workload's own context where the oracle's (untimed) prefill stays within ~10 s
    orc = O.DmtdOracle(ocfg, w, P + 64, dt)
    orc.prefill(di.make_prompts(sh.vocab, 1, prompt_len, seed=1)[0][:P])
    orc.decode_cycle(tau, n_late)
    t = time.perf_counter()
    n = 0
    cycles = 0
    while time.perf_counter() - t < 12.0 and orc.n_tok + tau < P + 60:
        n += len(orc.decode_cycle(tau, n_late))
        cycles += 1
    el = time.perf_counter() - t
    return {"value": round(n / el, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{cycles} cycles of tau={tau}, n_late={n_late} after a {P}-token prompt"
                      f"{'' if P == prompt_len else f' (the first {P} tokens of the {prompt_len}-token prompt)'}, "
                      f"batch 1 (one sequence of the workload), oracle in {'float32' if big else 'float64'}"}


if __name__ == "__main__":
    main()
